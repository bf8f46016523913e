// Stitched residual-add + bias + LayerNorm:
//     h = x (+ res) (+ bias);  mu = mean(h);  c = h - mu;  v = mean(c^2);
//     out = c * rsqrt(v + eps) (* gamma + beta)          -- one kernel, 12 ops
// This is the pattern of the paper's Figure 1 (Section 2.1) / Section 7.4: two row reductions and
// one expensive op on the per-row tensor, with every intermediate kept on chip.
//   * wave variant  (warp composition): an aligned group of L lanes of one wavefront
//     owns a row in registers; mean and variance are cross-lane all-reduces.
//   * block variant (block composition): a workgroup owns a row; per-wave partial
//     sums meet in LDS, the reduced values are read back from LDS by every thread.
// Two-pass variance on the register-resident row (no E[h^2] - mu^2 cancellation).
#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "kernel_table.hpp"
#include "row_skeleton.hpp"

namespace fsk {
using namespace fs;

// TI: dtype of x / res / bias / gamma / beta.  TO: dtype of out.  Both move VEC(TI)
// elements per lane per step, so the lane->column mapping is the same on both sides.
// FAST: residual, bias and affine all present, the row fills the lanes exactly and the
// row count fills the workgroups exactly, so every flag test, clamp and padding mask
// folds away at compile time (the shape of the benchmarked configuration).
template <typename TI, typename TO, int K, bool FAST>
struct LnRow {
  static constexpr int VEC = Elem<TI>::VEC;
  float h[K][VEC];
  u32x4 raw_gamma[K], raw_beta[K];   // fetched with the row, consumed after both reductions

  // All loads are issued before any value is used; vectors past the row end and rows
  // past the tensor end are clamped to a valid address and zeroed afterwards.
  __device__ __forceinline__ float load(const TI* __restrict__ x, const TI* __restrict__ res,
                                        const TI* __restrict__ bias, const TI* __restrict__ gamma,
                                        const TI* __restrict__ beta, const LayerNormP& p, uint32_t row,
                                        uint32_t lane, uint32_t stride) {
    const uint32_t nvec = p.cols / VEC;
    const bool has_res = FAST || p.has_res, has_bias = FAST || p.has_bias, has_affine = FAST || p.has_affine;
    const size_t base = (size_t)(FAST ? row : min(row, p.rows - 1)) * p.cols;
    auto vec_at = [&](int k) { return FAST ? lane + k * stride : min(lane + k * stride, nvec - 1); };
    u32x4 rx[K], rr[K], rb[K];
#pragma unroll
    for (int k = 0; k < K; ++k) rx[k] = load_raw_nt(x + base + vec_at(k) * VEC);
    if (has_res) {
#pragma unroll
      for (int k = 0; k < K; ++k) rr[k] = load_raw_nt(res + base + vec_at(k) * VEC);
    }
    if (has_bias) {
#pragma unroll
      for (int k = 0; k < K; ++k) rb[k] = load_raw(bias + vec_at(k) * VEC);
    }
    float sum = 0.0f;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      unpack(rx[k], h[k], (const TI*)nullptr);
      if (has_res) {
        float r[VEC];
        unpack(rr[k], r, (const TI*)nullptr);
#pragma unroll
        for (int e = 0; e < VEC; ++e) h[k][e] += r[e];
      }
      if (has_bias) {
        float b[VEC];
        unpack(rb[k], b, (const TI*)nullptr);
#pragma unroll
        for (int e = 0; e < VEC; ++e) h[k][e] += b[e];
      }
      if (!FAST && lane + k * stride >= nvec) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) h[k][e] = 0.0f;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) sum += h[k][e];
    }
    // gamma / beta are requested now, when the registers of the raw row are free again;
    // they arrive from cache while the two reductions run.
    if (has_affine) {
#pragma unroll
      for (int k = 0; k < K; ++k) {
        raw_gamma[k] = load_raw(gamma + vec_at(k) * VEC);
        raw_beta[k] = load_raw(beta + vec_at(k) * VEC);
      }
    }
    return sum;
  }

  __device__ __forceinline__ float center(const LayerNormP& p, float mean, uint32_t lane, uint32_t stride) {
    const uint32_t nvec = p.cols / VEC;
    float sq = 0.0f;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const float m = (FAST || lane + k * stride < nvec) ? mean : 0.0f;   // padded slots stay exactly zero
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        h[k][e] -= m;
        sq = __builtin_fmaf(h[k][e], h[k][e], sq);
      }
    }
    return sq;
  }

  __device__ __forceinline__ void finish(TO* __restrict__ out, const LayerNormP& p, uint32_t row,
                                         bool row_ok, uint32_t lane, uint32_t stride, float rstd) {
    const uint32_t nvec = p.cols / VEC;
    const size_t base = (size_t)row * p.cols;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const uint32_t j = lane + k * stride;
      if (FAST || p.has_affine) {
        float g[VEC], b[VEC];
        unpack(raw_gamma[k], g, (const TI*)nullptr);
        unpack(raw_beta[k], b, (const TI*)nullptr);
#pragma unroll
        for (int e = 0; e < VEC; ++e) h[k][e] = __builtin_fmaf(h[k][e] * rstd, g[e], b[e]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) h[k][e] *= rstd;
      }
      if (FAST || (row_ok && j < nvec)) StoreN<TO, VEC>::run(out + base + j * VEC, h[k]);
    }
  }
};

// STATS: the pattern also hands out the per-row mean and reciprocal standard deviation.  A template flag, not a
// run-time test of the pointers: the kernel without statistics must stay one basic block (see the file header).
template <typename TI, typename TO, int K, bool FAST, bool STATS>
__global__ void __launch_bounds__(256) k_layernorm_wave(const TI* __restrict__ x, const TI* __restrict__ res,
                                                        const TI* __restrict__ bias, const TI* __restrict__ gamma,
                                                        const TI* __restrict__ beta, TO* __restrict__ out,
                                                        float* __restrict__ mean_out, float* __restrict__ rstd_out,
                                                        LayerNormP p) {
  const uint32_t L = p.lanes_per_row;
  const uint32_t group = threadIdx.x >> p.lanes_log2;
  const uint32_t lane = threadIdx.x & (L - 1);
  const uint32_t row = blockIdx.x * (256u >> p.lanes_log2) + group;
  const bool row_ok = row < p.rows;
  const float inv_n = p.inv_cols;
  LnRow<TI, TO, K, FAST> r;
  const float mean = group_allreduce<OpSum>(r.load(x, res, bias, gamma, beta, p, row, lane, L), L) * inv_n;
  const float var = group_allreduce<OpSum>(r.center(p, mean, lane, L), L) * inv_n;
  const float rstd = fast_rsqrt(var + p.eps);
  r.finish(out, p, row, row_ok, lane, L, rstd);
  if constexpr (STATS) {
    if (row_ok && lane == 0) {
      if (mean_out) mean_out[row] = mean;
      if (rstd_out) rstd_out[row] = rstd;
    }
  }
}

template <typename TI, typename TO, int K, bool FAST>
__global__ void __launch_bounds__(256) k_layernorm_block(const TI* __restrict__ x, const TI* __restrict__ res,
                                                         const TI* __restrict__ bias, const TI* __restrict__ gamma,
                                                         const TI* __restrict__ beta, TO* __restrict__ out,
                                                         float* __restrict__ mean_out, float* __restrict__ rstd_out,
                                                         LayerNormP p) {
  __shared__ float slot_sum[2][4], slot_sq[2][4];
  const uint32_t n_waves = blockDim.x >> 6;
  const float inv_n = p.inv_cols;
  uint32_t it = 0;
  for (uint32_t row = blockIdx.x; row < p.rows; row += gridDim.x, ++it) {
    LnRow<TI, TO, K, FAST> r;
    // two slot sets alternate between rows: a wave may start row i+1 while a slower
    // one still reads the slots of row i.
    const float mean = block_allreduce<OpSum>(r.load(x, res, bias, gamma, beta, p, row, threadIdx.x, blockDim.x),
                                              slot_sum[it & 1], n_waves) * inv_n;
    const float var = block_allreduce<OpSum>(r.center(p, mean, threadIdx.x, blockDim.x),
                                             slot_sq[it & 1], n_waves) * inv_n;
    const float rstd = fast_rsqrt(var + p.eps);
    r.finish(out, p, row, true, threadIdx.x, blockDim.x, rstd);
    if constexpr (!FAST) {   // patterns with statistics use the general form of this kernel
      if (threadIdx.x == 0) {
        if (mean_out) mean_out[row] = mean;
        if (rstd_out) rstd_out[row] = rstd;
      }
    }
  }
}

// ---- LayerNorm backward ------------------------------------------------------------------
//   xh = (h - mu) rstd;  g = dy gamma;  dx = (g - mean(g) - xh mean(g xh)) rstd
//   dgamma = colsum(dy xh);  dbeta = colsum(dy)                      -- 13 ops, one launch + fold
// Row part: warp composition as in the forward kernel (two row reductions, issued
// together).  Column part: a lane keeps the column sums of the rows it has seen in
// registers while its lane group walks rows g, g + G, ... (software pipelined); the
// lane groups of a workgroup meet in LDS (regional step) and each workgroup leaves one
// [2, cols] row of partials for the fold launch (global step).
// A workgroup of WAVES wavefronts = G lane groups handles tiles of G*R consecutive rows
// (lane group g takes rows g, g+G, ... of the tile); the R rows of a lane group are all
// requested before the first is used.  With one tile per workgroup the whole problem
// runs as a single round of resident wavefronts, like the forward kernel; with more
// tiles than workgroups the column sums simply keep accumulating.
// FAST: the row fills the lanes exactly and the tiles fill the workgroups' rounds exactly.  Then nothing in the
// row loop is conditional, the next tile's loads are issued before this tile's arithmetic (software pipeline),
// and -- because the stores sit in no branch -- the wait for those loads leaves this tile's stores in flight.
template <typename T, int K, int R, int WAVES, bool FAST>
__global__ void __launch_bounds__(WAVES * 64) k_layernorm_bwd(const T* __restrict__ h, const T* __restrict__ dy,
                                                              const T* __restrict__ gamma, const float* __restrict__ mu,
                                                              const float* __restrict__ rstd, T* __restrict__ dx,
                                                              float* __restrict__ partials, LnBwdP p) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr uint32_t NT = WAVES * 64;
  extern __shared__ __align__(16) float lds[];         // [groups][2][cols]
  const uint32_t L = p.lanes_per_row;
  const uint32_t groups = NT >> p.lanes_log2;
  const uint32_t group = threadIdx.x >> p.lanes_log2, lane = threadIdx.x & (L - 1);
  const uint32_t nvec = p.cols / VEC;
  auto vec_at = [&](int k) { return FAST ? lane + k * L : min(lane + k * L, nvec - 1); };
  auto valid = [&](int k) { return FAST || lane + k * L < nvec; };

  float gam[K][VEC], dg[K][VEC], db[K][VEC];
  {
    u32x4 rg[K];
#pragma unroll
    for (int k = 0; k < K; ++k) rg[k] = load_raw(gamma + vec_at(k) * VEC);
#pragma unroll
    for (int k = 0; k < K; ++k) {
      unpack(rg[k], gam[k], (const T*)nullptr);
#pragma unroll
      for (int e = 0; e < VEC; ++e) { dg[k][e] = 0.0f; db[k][e] = 0.0f; }
    }
  }
  const uint32_t tile_rows = groups * R;
  const uint32_t n_tiles = (p.rows + tile_rows - 1) / tile_rows;
  struct Raw {
    u32x4 h[R][K], d[R][K];
    float mu[R], rs[R];
  };
  auto issue = [&](uint32_t tile, Raw& w) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint32_t row = tile * tile_rows + r * groups + group;
      const uint32_t rc = FAST ? row : min(row, p.rows - 1);
      const size_t base = (size_t)rc * p.cols;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        w.h[r][k] = load_raw_nt(h + base + vec_at(k) * VEC);
        w.d[r][k] = load_raw_nt(dy + base + vec_at(k) * VEC);
      }
      w.mu[r] = mu[rc];
      w.rs[r] = rstd[rc];
    }
  };
  auto compute = [&](uint32_t tile, const Raw& w) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint32_t row = tile * tile_rows + r * groups + group;
      const bool row_ok = FAST || row < p.rows;
      float xh[K][VEC], g[K][VEC];
      float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float dv[VEC];
        unpack(w.h[r][k], xh[k], (const T*)nullptr);
        unpack(w.d[r][k], dv, (const T*)nullptr);
        const bool ok = row_ok && valid(k);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float d = ok ? dv[e] : 0.0f;             // padding and past-the-end rows contribute nothing
          xh[k][e] = (xh[k][e] - w.mu[r]) * w.rs[r];
          g[k][e] = d * gam[k][e];
          s1 += g[k][e];
          s2 = __builtin_fmaf(g[k][e], xh[k][e], s2);
          dg[k][e] = __builtin_fmaf(d, xh[k][e], dg[k][e]);
          db[k][e] += d;
        }
      }
      const float m1 = group_allreduce<OpSum>(s1, (int)L) * p.inv_cols;
      const float m2 = group_allreduce<OpSum>(s2, (int)L) * p.inv_cols;
      const size_t base = (size_t)(FAST ? row : min(row, p.rows - 1)) * p.cols;
#pragma unroll
      for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) g[k][e] = (g[k][e] - m1 - xh[k][e] * m2) * w.rs[r];
        if (row_ok && valid(k)) store_vec_nt(dx + base + (lane + k * L) * VEC, g[k]);
      }
    }
  };
  if constexpr (FAST) {
    // n_tiles / gridDim.x rounds for every workgroup; first and last stand outside the loop so that the loop is
    // entered with the same loads and stores in flight that its own rounds leave behind
    Raw next;
    uint32_t tile = blockIdx.x;
    auto round = [&](uint32_t at) {
      const Raw cur = next;
      issue(at + gridDim.x, next);
      compute(at, cur);
    };
    issue(tile, next);
    if (tile + gridDim.x < n_tiles) {
      round(tile);
      tile += gridDim.x;
      for (; tile + gridDim.x < n_tiles; tile += gridDim.x) round(tile);
    }
    compute(tile, next);
  } else {
    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
      Raw w;
      issue(tile, w);
      compute(tile, w);
    }
  }
  // regional step: lane groups of the workgroup meet in LDS, folded in group order
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (valid(k)) {
      float* a = lds + (size_t)(group * 2) * p.cols + (lane + k * L) * VEC;
#pragma unroll
      for (int e = 0; e < VEC; e += 4) {   // 128-bit LDS stores: scalar ones would be VEC floats apart from lane to lane
        *reinterpret_cast<f32x4*>(a + e) = f32x4{dg[k][e], dg[k][e + 1], dg[k][e + 2], dg[k][e + 3]};
        *reinterpret_cast<f32x4*>(a + p.cols + e) = f32x4{db[k][e], db[k][e + 1], db[k][e + 2], db[k][e + 3]};
      }
    }
  }
  __syncthreads();
  float* prow = partials + (size_t)blockIdx.x * 2 * p.cols;
  for (uint32_t c = threadIdx.x; c < 2 * p.cols; c += NT) {
    float s = lds[c];
    for (uint32_t gi = 1; gi < groups; ++gi) s += lds[(size_t)gi * 2 * p.cols + c];
    prow[c] = s;
  }
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <typename T, int R, int WAVES, bool FAST>
const void* ln_bwd_sym_k(int K) {
  switch (K) {
    case 1: return (const void*)k_layernorm_bwd<T, 1, R, WAVES, FAST>;
    case 2: return (const void*)k_layernorm_bwd<T, 2, R, WAVES, FAST>;
    case 3: return (const void*)k_layernorm_bwd<T, 3, R, WAVES, FAST>;
    case 4: return (const void*)k_layernorm_bwd<T, 4, R, WAVES, FAST>;
    case 6: return (const void*)k_layernorm_bwd<T, 6, R, WAVES, FAST>;
    default: return nullptr;
  }
}
template <typename T, bool FAST>
const void* ln_bwd_sym_f(const LnBwdP& b) {
  if (b.waves == 4 && b.rows_per_group == 1) return ln_bwd_sym_k<T, 1, 4, FAST>(b.vecs_per_lane);
  if (b.waves == 4 && b.rows_per_group == 2) return ln_bwd_sym_k<T, 2, 4, FAST>(b.vecs_per_lane);
  if (b.waves == 4 && b.rows_per_group == 4) return ln_bwd_sym_k<T, 4, 4, FAST>(b.vecs_per_lane);
  if (b.waves == 8 && b.rows_per_group == 1) return ln_bwd_sym_k<T, 1, 8, FAST>(b.vecs_per_lane);
  if (b.waves == 8 && b.rows_per_group == 2) return ln_bwd_sym_k<T, 2, 8, FAST>(b.vecs_per_lane);
  return nullptr;
}
template <typename T>
const void* ln_bwd_sym(const LnBwdP& b) {
  return b.fast ? ln_bwd_sym_f<T, true>(b) : ln_bwd_sym_f<T, false>(b);
}
template <typename TI, typename TO>
const void* ln_sym(int32_t kernel, int K, bool fast, bool stats) {
#define FS_LN_CASE(KK)                                                                                     \
  case KK:                                                                                                 \
    if (kernel == K_LAYERNORM_WAVE) {                                                                      \
      if (stats) return fast ? (const void*)k_layernorm_wave<TI, TO, KK, true, true>                       \
                             : (const void*)k_layernorm_wave<TI, TO, KK, false, true>;                     \
      return fast ? (const void*)k_layernorm_wave<TI, TO, KK, true, false>                                 \
                  : (const void*)k_layernorm_wave<TI, TO, KK, false, false>;                               \
    }                                                                                                      \
    return fast && !stats ? (const void*)k_layernorm_block<TI, TO, KK, true>                               \
                          : (const void*)k_layernorm_block<TI, TO, KK, false>;
  switch (K) {
    FS_LN_CASE(1) FS_LN_CASE(2) FS_LN_CASE(3) FS_LN_CASE(4) FS_LN_CASE(6) FS_LN_CASE(8)
    default: return nullptr;
  }
#undef FS_LN_CASE
}
}  // namespace

const void* layernorm_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  if (kernel == K_LAYERNORM_BWD) {
    const LnBwdP& b = a.u.lnbwd;
    switch (b.dt) {
      case DT_F32: return ln_bwd_sym<float>(b);
      case DT_F16: return ln_bwd_sym<f16_t>(b);
      default: return ln_bwd_sym<bf16_t>(b);
    }
  }
  const LayerNormP& p = a.u.layernorm;
  const int K = p.vecs_per_lane;
  if (p.in_dt == DT_F32 && p.out_dt == DT_F32) return ln_sym<float, float>(kernel, K, p.fast != 0, p.stats != 0);
  if (p.in_dt == DT_F32 && p.out_dt == DT_BF16) return ln_sym<float, bf16_t>(kernel, K, p.fast != 0, p.stats != 0);
  if (p.in_dt == DT_F32 && p.out_dt == DT_F16) return ln_sym<float, f16_t>(kernel, K, p.fast != 0, p.stats != 0);
  if (p.in_dt == DT_BF16 && p.out_dt == DT_BF16) return ln_sym<bf16_t, bf16_t>(kernel, K, p.fast != 0, p.stats != 0);
  if (p.in_dt == DT_F16 && p.out_dt == DT_F16) return ln_sym<f16_t, f16_t>(kernel, K, p.fast != 0, p.stats != 0);
  return nullptr;
}

}  // namespace fs
