// Per-op baseline: one kernel per op of the subgraph, every intermediate through
// HBM as float32.  This is what the stitched kernels are measured against
// (the paper's un-stitched execution, Section 2.2: one launch and one round trip
// through off-chip memory per op).  Each kernel still uses 128-bit accesses where
// the shape allows, so the baseline is an honest one.
#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "kernel_table.hpp"

namespace fsk {
using namespace fs;

// ---- run-time-dtype vector access (dtype is wave-uniform, branches are scalar) ----
template <int V>
__device__ __forceinline__ void load_rt(const void* base, int dt, uint32_t off, float (&v)[V]) {
  if constexpr (V == 1) {
    if (dt == DT_F32) v[0] = load1(reinterpret_cast<const float*>(base) + off);
    else if (dt == DT_F16) v[0] = load1(reinterpret_cast<const f16_t*>(base) + off);
    else v[0] = load1(reinterpret_cast<const bf16_t*>(base) + off);
  } else if constexpr (V == 4) {
    if (dt == DT_F32) load_vec4(reinterpret_cast<const float*>(base) + off, v);
    else if (dt == DT_F16) load_vec4(reinterpret_cast<const f16_t*>(base) + off, v);
    else load_vec4(reinterpret_cast<const bf16_t*>(base) + off, v);
  } else {
    static_assert(V == 8, "vector width");
    if (dt == DT_F32) {
      float a[4], b[4];
      load_vec(reinterpret_cast<const float*>(base) + off, a);
      load_vec(reinterpret_cast<const float*>(base) + off + 4, b);
#pragma unroll
      for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
    } else if (dt == DT_F16) {
      load_vec(reinterpret_cast<const f16_t*>(base) + off, v);
    } else {
      load_vec(reinterpret_cast<const bf16_t*>(base) + off, v);
    }
  }
}

template <int V>
__device__ __forceinline__ void store_rt(void* base, int dt, uint32_t off, const float (&v)[V]) {
  if constexpr (V == 1) {
    if (dt == DT_F32) store1(reinterpret_cast<float*>(base) + off, v[0]);
    else if (dt == DT_F16) store1(reinterpret_cast<f16_t*>(base) + off, v[0]);
    else store1(reinterpret_cast<bf16_t*>(base) + off, v[0]);
  } else if constexpr (V == 4) {
    if (dt == DT_F32) store_vec4(reinterpret_cast<float*>(base) + off, v);
    else if (dt == DT_F16) store_vec4(reinterpret_cast<f16_t*>(base) + off, v);
    else store_vec4(reinterpret_cast<bf16_t*>(base) + off, v);
  } else {
    if (dt == DT_F32) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = v[i]; b[i] = v[4 + i]; }
      store_vec(reinterpret_cast<float*>(base) + off, a);
      store_vec(reinterpret_cast<float*>(base) + off + 4, b);
    } else if (dt == DT_F16) {
      store_vec(reinterpret_cast<f16_t*>(base) + off, v);
    } else {
      store_vec(reinterpret_cast<bf16_t*>(base) + off, v);
    }
  }
}

__device__ __forceinline__ float load_rt1(const void* base, int dt, uint32_t off) {
  float v[1];
  load_rt<1>(base, dt, off, v);
  return v[0];
}

// ---- unary ----------------------------------------------------------------------
__device__ __forceinline__ float unary_apply(int op, float x, float value) {
  switch (op) {
    case U_SCALE: return x * value;
    case U_ADD_SCALAR: return x + value;
    case U_SQUARE: return x * x;
    case U_EXP: return fast_exp(x);
    case U_RSQRT: return fast_rsqrt(x);
    case U_TANH: return tanhf(x);
    case U_GELU: return gelu_fwd(x);
    case U_GELU_GRAD: return gelu_grad(x);
    case U_LOG: return full_log(x);
    case U_SIGMOID: return fast_sigmoid(x);
    case U_RELU: return fmaxf(x, 0.0f);
    case U_ABS: return __builtin_fabsf(x);
    case U_SQRT: return full_sqrt(x);
    default: return x;
  }
}

template <int V>
__global__ void __launch_bounds__(256) k_unary(const void* in, void* out, UnaryP p) {
  const uint32_t i = (blockIdx.x * 256u + threadIdx.x) * V;
  if (i >= p.n) return;
  float v[V];
  load_rt<V>(in, p.in_dt, i, v);
#pragma unroll
  for (int k = 0; k < V; ++k) v[k] = unary_apply(p.op, v[k], p.value);
  store_rt<V>(out, p.out_dt, i, v);
}

// ---- binary with broadcasting ---------------------------------------------------
__device__ __forceinline__ float binary_apply(int op, float a, float b) {
  switch (op) {
    case B_ADD: return a + b;
    case B_SUB: return a - b;
    case B_MUL: return a * b;
    case B_DIV: return a / b;
    case B_MAX: return fmaxf(a, b);
    default: return a;
  }
}

template <int V>
__global__ void __launch_bounds__(256) k_binary(const void* a, const void* b, void* out, BinaryP p) {
  const uint32_t e = (blockIdx.x * 256u + threadIdx.x) * V;
  if (e >= p.n) return;
  // coordinates of element e in the collapsed output, innermost first
  uint32_t rest = e, oa = 0, ob = 0;
  uint32_t inner_sa = p.sa[p.rank - 1], inner_sb = p.sb[p.rank - 1];
  for (int k = p.rank - 1; k >= 0; --k) {
    uint32_t c;
    if (k == 0) { c = rest; }
    else { c = rest % p.dims[k]; rest = rest / p.dims[k]; }
    oa += c * p.sa[k];
    ob += c * p.sb[k];
  }
  float va[V], vb[V];
  if (inner_sa == 1 || V == 1) load_rt<V>(a, p.a_dt, oa, va);
  else { float s = load_rt1(a, p.a_dt, oa);
#pragma unroll
         for (int k = 0; k < V; ++k) va[k] = s; }
  if (inner_sb == 1 || V == 1) load_rt<V>(b, p.b_dt, ob, vb);
  else { float s = load_rt1(b, p.b_dt, ob);
#pragma unroll
         for (int k = 0; k < V; ++k) vb[k] = s; }
#pragma unroll
  for (int k = 0; k < V; ++k) va[k] = binary_apply(p.op, va[k], vb[k]);
  store_rt<V>(out, p.out_dt, e, va);
}

// ---- row reduction: [rows, cols] -> [rows] --------------------------------------
__device__ __forceinline__ float red_identity(int op) { return op == R_MAX ? -INFINITY : 0.0f; }
__device__ __forceinline__ float red_apply(int op, float a, float b) { return op == R_MAX ? fmaxf(a, b) : a + b; }

template <int V>
__global__ void __launch_bounds__(256) k_reduce_row(const void* in, void* out, ReduceP p) {
  const uint32_t L = p.lanes_per_row;
  const uint32_t rows_per_block = 256u / L;
  const uint32_t row = blockIdx.x * rows_per_block + threadIdx.x / L;
  const uint32_t lane = threadIdx.x % L;
  float acc = red_identity(p.op);
  if (row < p.outer) {
    const uint32_t base = row * p.red;
    for (uint32_t c = lane * V; c < p.red; c += L * V) {
      float v[V];
      load_rt<V>(in, p.in_dt, base + c, v);
#pragma unroll
      for (int k = 0; k < V; ++k) acc = red_apply(p.op, acc, v[k]);
    }
  }
  acc = (p.op == R_MAX) ? group_allreduce<OpMax>(acc, L) : group_allreduce<OpSum>(acc, L);
  if (row < p.outer && lane == 0) {
    float r[1] = {acc * p.post_scale};
    store_rt<1>(out, p.out_dt, row, r);
  }
}

// ---- reduction over a middle axis: [outer, red, inner] -> [outer, nchunk, inner] --
// Each lane owns V adjacent inner positions and walks `chunk` rows of the reduced
// axis; lanes of a wave read adjacent addresses.  A second launch of the same
// kernel folds the chunks.
template <int V>
__global__ void __launch_bounds__(256) k_reduce_mid(const void* in, void* out, ReduceP p) {
  const uint32_t inner_vecs = p.inner / V;
  const uint32_t n_inner_blocks = (inner_vecs + 255u) / 256u;
  uint32_t bid = blockIdx.x;
  const uint32_t ib = bid % n_inner_blocks; bid /= n_inner_blocks;
  const uint32_t ch = bid % p.nchunk;
  const uint32_t o = bid / p.nchunk;
  const uint32_t iv = ib * 256u + threadIdx.x;
  if (iv >= inner_vecs) return;
  const uint32_t r0 = ch * p.chunk;
  const uint32_t r1 = min(r0 + p.chunk, p.red);
  float acc[V];
#pragma unroll
  for (int k = 0; k < V; ++k) acc[k] = red_identity(p.op);
  uint32_t off = (o * p.red + r0) * p.inner + iv * V;
  for (uint32_t r = r0; r < r1; ++r, off += p.inner) {
    float v[V];
    load_rt<V>(in, p.in_dt, off, v);
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = red_apply(p.op, acc[k], v[k]);
  }
#pragma unroll
  for (int k = 0; k < V; ++k) acc[k] *= p.post_scale;
  store_rt<V>(out, p.out_dt, (o * p.nchunk + ch) * p.inner + iv * V, acc);
}

// ---- transpose, innermost axis kept: rows of contiguous elements are re-ordered ----
template <typename VT>
__global__ void __launch_bounds__(256) k_transpose_rows(const void* in, void* out, TransposeP p) {
  const uint32_t vi = blockIdx.x * 256u + threadIdx.x;   // vector index in the output
  const uint32_t e = vi * p.vec;
  if (e >= p.n) return;
  uint32_t rest = e;
  const uint32_t c3 = rest % p.out_dims[3]; rest /= p.out_dims[3];
  const uint32_t c2 = rest % p.out_dims[2]; rest /= p.out_dims[2];
  const uint32_t c1 = rest % p.out_dims[1];
  const uint32_t c0 = rest / p.out_dims[1];
  const uint32_t src = c0 * p.in_stride[0] + c1 * p.in_stride[1] + c2 * p.in_stride[2] + c3;
  reinterpret_cast<VT*>(out)[vi] = reinterpret_cast<const VT*>(in)[src / p.vec];
}

// ---- transpose, innermost axis moves: 32x32 tile through padded LDS ---------------
// Tile rows run along the output position q that receives the input's innermost
// axis; tile columns run along the output's innermost axis.  Reads are contiguous
// along the input's innermost axis, writes along the output's; the 33-word pitch
// keeps both LDS phases free of bank conflicts.
template <typename T>
__global__ void __launch_bounds__(256) k_transpose_tile(const T* __restrict__ in, T* __restrict__ out, TransposeP p) {
  __shared__ T tile[32][33];
  const uint32_t q = p.tile_in_axis_out_pos;
  const uint32_t nq = p.out_dims[q], n3 = p.out_dims[3];
  const uint32_t tq = (nq + 31u) / 32u, t3 = (n3 + 31u) / 32u;
  uint32_t bid = blockIdx.x;
  const uint32_t b3 = bid % t3; bid /= t3;
  const uint32_t bq = bid % tq; bid /= tq;
  // the two remaining output axes form the batch index
  uint32_t ax[2], na = 0;
  for (uint32_t k = 0; k < 3; ++k) if (k != q) ax[na++] = k;
  const uint32_t cb1 = bid % p.out_dims[ax[1]];
  const uint32_t cb0 = bid / p.out_dims[ax[1]];
  const uint32_t in_base = cb0 * p.in_stride[ax[0]] + cb1 * p.in_stride[ax[1]];
  const uint32_t out_base = cb0 * p.out_stride[ax[0]] + cb1 * p.out_stride[ax[1]];
  const uint32_t tx = threadIdx.x & 31u, ty = threadIdx.x >> 5;
  // read: tx along input-innermost (output axis q), ty along output-innermost
  for (uint32_t j = ty; j < 32u; j += 8u) {
    const uint32_t cq = bq * 32u + tx, c3 = b3 * 32u + j;
    if (cq < nq && c3 < n3) tile[j][tx] = in[in_base + cq + c3 * p.in_stride[3]];
  }
  __syncthreads();
  // write: tx along output-innermost, ty along output axis q
  for (uint32_t i = ty; i < 32u; i += 8u) {
    const uint32_t cq = bq * 32u + i, c3 = b3 * 32u + tx;
    if (cq < nq && c3 < n3) out[out_base + cq * p.out_stride[q] + c3] = tile[tx][i];
  }
}

// ---- transpose, innermost axis moves: 128-bit accesses on both HBM sides AND both LDS sides ----------------
// The tile is UQ x U3 units of VEC x VEC elements (UQ * U3 = 256 threads, one unit each; VEC = elements in 16
// bytes), TQ = UQ * VEC along the input's innermost axis (output axis q) by T3 = U3 * VEC along the output's.
// A thread loads its unit as VEC rows of 16 bytes (a wave reads runs of UQ * 16 bytes), transposes it in
// registers (32-bit elements: a renaming; 16-bit elements: one byte-permute per pair), and parks it in LDS as VEC
// 16-byte pieces, one per tile column, each holding VEC consecutive elements of the OUTPUT's innermost axis.
// After the barrier a thread reads one 16-byte piece per pass and stores it: a wave writes runs of U3 * 16 bytes
// (or several full columns).  LDS is [TQ columns][U3 pieces] of 16 bytes, unpadded; piece u of column c sits at
// position u ^ (c / VEC mod 8): any eight neighbouring lanes -- the lanes one LDS cycle serves for a 128-bit
// access -- then hit eight different 16-byte bank groups, writing (same row unit, eight column units) and
// reading (same column, eight neighbouring pieces) alike, where a padded tile with scalar accesses ran at two
// lanes per bank (measured: conflict cycles half of the LDS-active cycles).
// Needs both tile axes to be multiples of VEC; other shapes use the 32x32 scalar kernel.
template <typename T, int UQ>
__global__ void __launch_bounds__(256) k_transpose_tile64(const T* __restrict__ in, T* __restrict__ out, TransposeP p) {
  constexpr uint32_t VEC = 16 / sizeof(T), U3 = 256 / UQ, TQ = UQ * VEC, T3 = U3 * VEC;
  __shared__ u32x4 tile[TQ * U3];
  const uint32_t q = p.tile_in_axis_out_pos;
  const uint32_t nq = p.out_dims[q], n3 = p.out_dims[3];
  const uint32_t tq = (nq + TQ - 1) / TQ, t3 = (n3 + T3 - 1) / T3;
  uint32_t bid = blockIdx.x;
  uint32_t ax[2], na = 0;
  for (uint32_t k = 0; k < 3; ++k) if (k != q) ax[na++] = k;
  uint32_t b3, bq, cb1, cb0;
  if (p.order == 0) {
    b3 = bid % t3; bid /= t3;
    bq = bid % tq; bid /= tq;
    cb1 = bid % p.out_dims[ax[1]];
    cb0 = bid / p.out_dims[ax[1]];
  } else {
    cb1 = bid % p.out_dims[ax[1]]; bid /= p.out_dims[ax[1]];
    b3 = bid % t3; bid /= t3;
    bq = bid % tq;
    cb0 = bid / tq;
  }
  const uint32_t in_base = cb0 * p.in_stride[ax[0]] + cb1 * p.in_stride[ax[1]];
  const uint32_t out_base = cb0 * p.out_stride[ax[0]] + cb1 * p.out_stride[ax[1]];
  // load: unit (uq, u3) = columns uq*VEC.. of rows u3*VEC..; padding units are clamped to valid addresses (what
  // they park in LDS is never stored)
  const uint32_t uq = threadIdx.x % UQ, u3 = threadIdx.x / UQ;
  const uint32_t cq0 = min(bq * TQ + uq * VEC, nq - VEC), c30 = min(b3 * T3 + u3 * VEC, n3 - VEC);
  u32x4 row[VEC];
#pragma unroll
  for (uint32_t s = 0; s < VEC; ++s)
    row[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in + in_base + cq0 + (size_t)(c30 + s) * p.in_stride[3]));
  // transpose in registers: col[e] = elements e of rows 0..VEC-1
  u32x4 col[VEC];
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (uint32_t e = 0; e < 4; ++e) col[e] = u32x4{row[0][e], row[1][e], row[2][e], row[3][e]};
  } else {
    // 2x2 blocks of 16-bit elements first: for rows (2m, 2m+1) and dword k, lo = [r0.lo16, r1.lo16] is column 2k,
    // hi = [r0.hi16, r1.hi16] column 2k+1, each holding rows 2m, 2m+1; the rest is a renaming
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
      uint32_t lo[4], hi[4];
#pragma unroll
      for (uint32_t m = 0; m < 4; ++m) {
        lo[m] = __builtin_amdgcn_perm(row[2 * m + 1][k], row[2 * m][k], 0x05040100u);   // [r0.lo, r1.lo]
        hi[m] = __builtin_amdgcn_perm(row[2 * m + 1][k], row[2 * m][k], 0x07060302u);   // [r0.hi, r1.hi]
      }
      col[2 * k] = u32x4{lo[0], lo[1], lo[2], lo[3]};
      col[2 * k + 1] = u32x4{hi[0], hi[1], hi[2], hi[3]};
    }
  }
#pragma unroll
  for (uint32_t e = 0; e < VEC; ++e) {
    const uint32_t c = uq * VEC + e;
    tile[c * U3 + (u3 ^ (uq & 7u))] = col[e];
  }
  __syncthreads();
  // store: piece u of column c -> 16 bytes of output row (bq*TQ + c) at column b3*T3 + u*VEC
  const uint32_t u = threadIdx.x % U3, c_first = threadIdx.x / U3;
#pragma unroll
  for (uint32_t s = 0; s < TQ / UQ; ++s) {
    const uint32_t c = c_first + s * UQ;
    const u32x4 v = tile[c * U3 + (u ^ ((c / VEC) & 7u))];
    const uint32_t cq = bq * TQ + c, c3 = b3 * T3 + u * VEC;
    if (cq < nq && c3 < n3) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + out_base + (size_t)cq * p.out_stride[q] + c3));
  }
}

// ---- streaming copy (the measured HBM ceiling) ------------------------------------
__global__ void __launch_bounds__(256) k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, UnaryP p) {
  const uint32_t n_vec = p.n;   // 128-bit vectors
  uint32_t i = blockIdx.x * 1024u + threadIdx.x;
  u32x4 v[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) if (i + k * 256u < n_vec) v[k] = __builtin_nontemporal_load(src + i + k * 256u);
#pragma unroll
  for (int k = 0; k < 4; ++k) if (i + k * 256u < n_vec) __builtin_nontemporal_store(v[k], dst + i + k * 256u);
}

}  // namespace fsk

// ---- host launchers ----------------------------------------------------------------
namespace fs {
using namespace fsk;

const void* unfused_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  switch (kernel) {
    case K_UNARY:
      return a.u.unary.vec == 8 ? (const void*)k_unary<8> : a.u.unary.vec == 4 ? (const void*)k_unary<4> : (const void*)k_unary<1>;
    case K_BINARY:
      return a.u.binary.vec == 8 ? (const void*)k_binary<8> : a.u.binary.vec == 4 ? (const void*)k_binary<4> : (const void*)k_binary<1>;
    case K_REDUCE_ROW:
      return a.u.reduce.vec == 8 ? (const void*)k_reduce_row<8> : a.u.reduce.vec == 4 ? (const void*)k_reduce_row<4> : (const void*)k_reduce_row<1>;
    case K_REDUCE_MID:
      return a.u.reduce.vec == 8 ? (const void*)k_reduce_mid<8> : a.u.reduce.vec == 4 ? (const void*)k_reduce_mid<4> : (const void*)k_reduce_mid<1>;
    case K_TRANSPOSE_ROWS: {
      const int vb = a.u.transpose.vec * a.u.transpose.elem_bytes;
      return vb == 16 ? (const void*)k_transpose_rows<u32x4> : vb == 8 ? (const void*)k_transpose_rows<u32x2>
           : vb == 4 ? (const void*)k_transpose_rows<uint32_t> : (const void*)k_transpose_rows<uint16_t>;
    }
    case K_TRANSPOSE_TILE:
      if (a.u.transpose.vec > 1) {
        if (a.u.transpose.tile_uq == 8)
          return a.u.transpose.elem_bytes == 4 ? (const void*)k_transpose_tile64<uint32_t, 8> : (const void*)k_transpose_tile64<uint16_t, 8>;
        return a.u.transpose.elem_bytes == 4 ? (const void*)k_transpose_tile64<uint32_t, 16> : (const void*)k_transpose_tile64<uint16_t, 16>;
      }
      return a.u.transpose.elem_bytes == 4 ? (const void*)k_transpose_tile<uint32_t> : (const void*)k_transpose_tile<uint16_t>;
    case K_COPY:
      return (const void*)k_copy;
    default:
      return nullptr;
  }
}

}  // namespace fs
