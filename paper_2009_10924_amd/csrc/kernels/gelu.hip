// Stitched bias + tanh-GELU, alone (thread composition) or packed with the
// bias-gradient column reduction (kernel packing + a global hand-off):
//     z = x + bias;  y = gelu(z);  dbias = colsum(grad * gelu'(z))
// GELU and GELU' share one exp and one reciprocal per element (the computation-reuse
// rule of the paper's Section 4.5) and one read of x.
//
// The column reduction needs rows owned by other workgroups, which the paper's
// schemes exclude (Section 4.1, last paragraph: no inter-block communication).  Here
// it is one round trip through device memory: every workgroup leaves its column
// partials in a [n_row_blocks, cols] float32 workspace, and the partials are folded in
// row-block order (fixed order: results are bit-identical from run to run) by a second,
// tiny launch (k_colfold): the kernel boundary is the hand-off.  Folding inside the same
// launch (the workgroup that arrives last reads the others' partials) needs an agent-scope
// release per workgroup before it signals its arrival, which on this part writes back the
// whole L2 of the workgroup's die while that cache is full of freshly stored y: measured
// at 1.6x the time of the two launches, so that form is not built.
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
  const u32x4 rx = load_raw_nt(x + (size_t)vi * VEC);
  const u32x4 rb = load_raw(bias + cv * VEC);
  float v[VEC], b[VEC];
  unpack(rx, v, (const T*)nullptr);
  unpack(rb, b, (const T*)nullptr);
#pragma unroll
  for (int e = 0; e < VEC; ++e) v[e] = gelu_fwd(v[e] + b[e]);
  store_vec_nt(y + (size_t)vi * VEC, v);
}

// y = gelu(z) and acc += g * gelu'(z) with shared sub-expressions:
//   t = -2c log2(e) (1 + a z^2);  e = 2^(z t) = exp(-2u);  s = 1/(1+e);  y = z s
//   gelu' = s + z s (1-s) d(2u)/dz,   d(2u)/dz = 2c (1 + 3 a z^2)
__device__ __forceinline__ float gelu_and_grad(float z, float g, float& acc) {
  constexpr float c = 0.7978845608028654f, a = 0.044715f;
  constexpr float k = -2.0f * c * kLog2e;
  const float z2 = z * z;
  const float t = __builtin_fmaf(k * a, z2, k);
  const float s = fast_rcp(1.0f + __builtin_amdgcn_exp2f(z * t));
  const float y = z * s;
  const float dw = __builtin_fmaf(6.0f * c * a, z2, 2.0f * c);
  acc = __builtin_fmaf(g, __builtin_fmaf(__builtin_fmaf(-y, s, y), dw, s), acc);
  return y;
}

// ---- bias + GELU forward + bias-gradient column partials ------------------------------
// Workgroup (ct, rb): column tile ct of 64*VEC columns, row tiles rb, rb + n_rb, ... of
// WAVES*UNROLL rows each.  Lane l owns columns [l*VEC, l*VEC+VEC) of the tile, wave w
// rows w, w+WAVES, ... of a row tile, so every wave-wide access is one contiguous
// 1 KB piece, and at any moment the resident workgroups sweep one band of rows
// (DRAM pages stay open) while each keeps its column sums in registers.
// FAST: the rows fill every workgroup's row tiles exactly and the columns fill the column
// tiles, so the row loop has no test inside.  That matters beyond the saved compares: the
// memory counter of this part counts loads and stores alike, in issue order, and when a
// store sits inside a branch the compiler can no longer tell how many stores follow the
// loads it waits for, so it waits for everything -- every round of the loop then ends
// with the wave idle until its own y stores are acknowledged.  With unconditional stores
// the wait before the next tile's data leaves the UNROLL stores of this tile in flight.
template <typename T, int WAVES, int UNROLL, bool FAST>
__global__ void __launch_bounds__(WAVES * 64) k_bias_gelu_dbias(const T* __restrict__ x, const T* __restrict__ bias,
                                                                const T* __restrict__ grad, T* __restrict__ y,
                                                                float* __restrict__ partials, GeluP p) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int TILE_COLS = 64 * VEC, NT = WAVES * 64, TILE_ROWS = WAVES * UNROLL;
  __shared__ __align__(16) float red[WAVES][TILE_COLS];
  const uint32_t n_col_tiles = (p.cols + TILE_COLS - 1) / TILE_COLS;
  const uint32_t rb = blockIdx.x / n_col_tiles;
  const uint32_t ct = blockIdx.x - rb * n_col_tiles;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t col = FAST ? ct * TILE_COLS + lane * VEC
                            : min(ct * TILE_COLS + lane * VEC, p.cols - VEC);   // clamped lanes of a ragged tile redo valid columns
  const bool col_ok = FAST || ct * TILE_COLS + lane * VEC < p.cols;

  float acc[VEC], b[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
  unpack(load_raw(bias + col), b, (const T*)nullptr);
  // software pipeline: the loads of the next row tile are in flight while this one is
  // computed, so a wave overlaps its own ALU phase (two quarter-rate ops per element)
  // with its own memory phase instead of relying on the other waves of the SIMD.
  u32x4 nx[UNROLL], ng[UNROLL];
  auto issue = [&](uint32_t r0) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const uint32_t r = r0 + wave + u * WAVES;
      const size_t off = (size_t)(FAST ? r : min(r, p.rows - 1)) * p.cols + col;
      nx[u] = load_raw_nt(x + off);
      ng[u] = load_raw_nt(grad + off);
    }
  };
  auto compute = [&](uint32_t r0, const u32x4 (&rx)[UNROLL], const u32x4 (&rg)[UNROLL]) {
    if constexpr (FAST) {
      // all rows of the tile first, then their stores in one burst (measured: 0.5 us of 50 against a store
      // after every row; the memory system takes a run of writes better than writes sprinkled between reads)
      float out[UNROLL][VEC];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        float gv[VEC];
        unpack(rx[u], out[u], (const T*)nullptr);
        unpack(rg[u], gv, (const T*)nullptr);
#pragma unroll
        for (int e = 0; e < VEC; ++e) out[u][e] = gelu_and_grad(out[u][e] + b[e], gv[e], acc[e]);
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) store_vec_nt(y + (size_t)(r0 + wave + u * WAVES) * p.cols + col, out[u]);
    } else {
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t r = r0 + wave + u * WAVES;
        if (r < p.rows) {
          float xv[VEC], gv[VEC];
          unpack(rx[u], xv, (const T*)nullptr);
          unpack(rg[u], gv, (const T*)nullptr);
#pragma unroll
          for (int e = 0; e < VEC; ++e) xv[e] = gelu_and_grad(xv[e] + b[e], gv[e], acc[e]);
          if (col_ok) store_vec_nt(y + (size_t)r * p.cols + col, xv);
        }
      }
    }
  };
  const uint32_t stride = p.n_row_tiles * TILE_ROWS;
  uint32_t r0 = rb * TILE_ROWS;
  if constexpr (FAST) {
    // every workgroup makes the same number of rounds (rows / stride >= 1), none with a test around its loads or
    // its stores.  First and last round stand outside the loop: the loop is then entered with the same sequence of
    // loads and stores in flight that its own rounds leave behind, which is what lets the wait at its head be
    // "all but the last stores" on both ways in.
    auto round = [&](uint32_t at) {
      u32x4 rx[UNROLL], rg[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) { rx[u] = nx[u]; rg[u] = ng[u]; }
      issue(at + stride);
      compute(at, rx, rg);
    };
    issue(r0);
    if (r0 + stride < p.rows) {
      round(r0);
      r0 += stride;
      for (; r0 + stride < p.rows; r0 += stride) round(r0);
    }
    compute(r0, nx, ng);
  } else {
    if (r0 < p.rows) issue(r0);
    for (; r0 < p.rows; r0 += stride) {
      u32x4 rx[UNROLL], rg[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) { rx[u] = nx[u]; rg[u] = ng[u]; }
      if (r0 + stride < p.rows) issue(r0 + stride);
      compute(r0, rx, rg);
    }
  }

  // regional step: fold the waves of this workgroup through LDS, in wave order
#pragma unroll
  for (int e = 0; e < VEC; e += 4)   // 128-bit LDS stores: scalar ones would be VEC floats apart from lane to lane
    *reinterpret_cast<f32x4*>(&red[wave][lane * VEC + e]) = f32x4{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
  __syncthreads();
  for (uint32_t c = threadIdx.x; c < TILE_COLS; c += NT) {
    float s = red[0][c];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) s += red[w][c];
    const uint32_t gc = ct * TILE_COLS + c;
    if (gc < p.cols) partials[(size_t)rb * p.cols + gc] = s;
  }
}

// ---- fold of column partials: [n_rows, width] float32 (rows `stride` floats apart) -> [width] ---------
// Workgroup = Q column quads x G row groups (256 threads).  Each thread sums its rows in
// order with eight independent loads in flight, LDS folds the G groups in order.  Few
// partial rows: (Q,G) = (16,16); many: (4,64), so a thread still needs one batch of loads.
template <int Q, int G>
__device__ __forceinline__ void fold_tile(const float* __restrict__ partials, float* __restrict__ out0, float* __restrict__ out1,
                                          uint32_t n, uint32_t width, uint32_t stride, uint32_t split, uint32_t block,
                                          f32x4* __restrict__ sm, int32_t out_dt) {
  const uint32_t q = threadIdx.x % Q, g = threadIdx.x / Q;
  const uint32_t col = (block * Q + q) * 4u;
  f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
  if (col < width) {
    uint32_t t = g;
    for (; t + 7 * G < n; t += 8 * G) {
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4*>(partials + (size_t)(t + u * G) * stride + col);
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; t < n; t += G) s += *reinterpret_cast<const f32x4*>(partials + (size_t)t * stride + col);
  }
  sm[g * Q + q] = s;
  __syncthreads();
  // the G row groups fold through LDS four at a time (G = 16: two levels, G = 64: three; the same order every
  // run): a barrier costs more than three more LDS reads, and a serial walk over all G slots more than both
#pragma unroll
  for (int span = G / 4; span >= 1; span /= 4) {
    if ((int)g < span) sm[g * Q + q] += sm[(g + span) * Q + q] + sm[(g + 2 * span) * Q + q] + sm[(g + 3 * span) * Q + q];
    __syncthreads();
  }
  if (g == 0 && col < width) {
    const f32x4 v = sm[q];
    // the split is a multiple of 4, so a quad never straddles the two outputs; sums handed out in 16 bits are
    // rounded here, once
    float* const base = col < split ? out0 : out1;
    const uint32_t at = col < split ? col : col - split;
    if (out_dt == DT_F32) {
      *reinterpret_cast<f32x4*>(base + at) = v;
    } else {
      const float quad[4] = {v.x, v.y, v.z, v.w};
      if (out_dt == DT_BF16) StoreN<bf16_t, 4>::run(reinterpret_cast<bf16_t*>(base) + at, quad);
      else StoreN<f16_t, 4>::run(reinterpret_cast<f16_t*>(base) + at, quad);
    }
  }
}

template <int Q, int G>
__global__ void __launch_bounds__(256) k_colfold(const float* __restrict__ partials, float* __restrict__ out0,
                                                 float* __restrict__ out1, GeluP p) {
  __shared__ f32x4 sm[G * Q];
  // stride >= width: a fold may take a slice of wider partial rows
  fold_tile<Q, G>(partials, out0, out1, p.n_row_tiles, p.fold_cols, p.cols, p.fold_split, blockIdx.x, sm, p.dt);
}

// Several independent folds in one launch: workgroups [first_block[i], first_block[i+1]) run fold i.  The table
// is read from the kernel-argument segment with wave-uniform addresses (indexing the by-value parameter would
// make the compiler copy it to per-lane scratch first).
typedef const FoldManyP __attribute__((address_space(4))) * ConstFolds;

__global__ void __launch_bounds__(256) k_colfold_many(const FoldManyP table_in_kernarg) {
  __shared__ f32x4 sm[256];
  ConstFolds tab = (ConstFolds)__builtin_amdgcn_kernarg_segment_ptr();
  const uint32_t b = blockIdx.x;
  int i = -1;
#pragma unroll
  for (int j = 0; j < kFoldManyMax; ++j) i += b >= tab->first_block[j] ? 1 : 0;   // first_block[0] = 0, unused ones ~0
  i = __builtin_amdgcn_readfirstlane(i);
  const float* partials = tab->partials[i];
  float* out0 = tab->out0[i];
  float* out1 = tab->out1[i];
  const uint32_t block = b - tab->first_block[i];
  if (tab->quads[i] == 4)
    fold_tile<4, 64>(partials, out0, out1, tab->n[i], tab->width[i], tab->stride[i], tab->split[i], block, sm, tab->out_dt[i]);
  else
    fold_tile<16, 16>(partials, out0, out1, tab->n[i], tab->width[i], tab->stride[i], tab->split[i], block, sm, tab->out_dt[i]);
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <typename T, bool FAST>
const void* dbias_sym(int waves, int unroll) {
  if (waves == 4 && unroll == 2) return (const void*)k_bias_gelu_dbias<T, 4, 2, FAST>;
  if (waves == 4 && unroll == 4) return (const void*)k_bias_gelu_dbias<T, 4, 4, FAST>;
  if (waves == 8 && unroll == 2) return (const void*)k_bias_gelu_dbias<T, 8, 2, FAST>;
  if (waves == 8 && unroll == 4) return (const void*)k_bias_gelu_dbias<T, 8, 4, FAST>;
  return nullptr;
}
template <typename T>
const void* gelu_sym(int32_t kernel, const GeluP& p) {
  if (kernel == K_BIAS_GELU) return (const void*)k_bias_gelu<T>;
  return p.fast ? dbias_sym<T, true>(p.waves, p.unroll) : dbias_sym<T, false>(p.waves, p.unroll);
}
}  // namespace

int launch_fold_many(const FoldManyP& table, uint32_t n_blocks, void* stream) {
  if (n_blocks == 0) return 0;
  FoldManyP t = table;
  void* argv[1] = {&t};
  return (int)hipLaunchKernel((const void*)k_colfold_many, dim3(n_blocks), dim3(256), argv, 0, static_cast<hipStream_t>(stream));
}

const void* gelu_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  const GeluP& p = a.u.gelu;
  if (kernel == K_COLFOLD) return p.fold_quads == 4 ? (const void*)k_colfold<4, 64> : (const void*)k_colfold<16, 16>;
  switch (p.dt) {
    case DT_F32: return gelu_sym<float>(kernel, p);
    case DT_F16: return gelu_sym<f16_t>(kernel, p);
    default: return gelu_sym<bf16_t>(kernel, p);
  }
}

}  // namespace fs
