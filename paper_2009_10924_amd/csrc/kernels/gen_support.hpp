// Support code of the generated row kernels (paper Section 4: the code generator takes a
// fusion pattern and produces one kernel).  A generated kernel is straight-line code over
// named per-lane values; what every such kernel shares -- the geometry of a row over a lane
// group or a workgroup, the 128-bit loads issued up front at clamped addresses, unpacking,
// the streaming store and the row reductions -- lives here, with every extent a template
// constant so that index arithmetic, padding tests and loops fold away at compile time.
// This header is embedded in the library as text and handed to the run-time compiler in
// front of the generated kernel; the library's own build also compiles it (a fixed sample
// kernel instantiates it) so that a mistake shows at build time.
#pragma once
#include "device_utils.hpp"

namespace fsk {

// Pointer block of a generated kernel, one by-value argument (slots as in K_ROW_PROGRAM).
struct GenArgs {
  const void* full[4];
  const void* col[4];
  const void* rscal[4];
  void* out[4];
  void* rout[4];
};

// ROWS x COLS row space; VEC elements per lane and step; K steps per lane; L lanes per row
// (a lane group of one wavefront), or the whole 256-thread workgroup when BLOCK.
template <uint32_t ROWS, uint32_t COLS, int VEC, int K, uint32_t L, bool BLOCK>
struct GenRow {
  static constexpr uint32_t NVEC = COLS / VEC;
  static constexpr uint32_t LANES = BLOCK ? 256u : L;
  static constexpr uint32_t ROWS_PER_WG = BLOCK ? 1u : 256u / L;
  // the row fills its lanes / the rows fill the workgroups: no clamp, no padding test
  static constexpr bool FULL_COLS = NVEC == LANES * K;
  static constexpr bool FULL_ROWS = ROWS % ROWS_PER_WG == 0;
  static constexpr int KV = K * VEC;

  uint32_t lane, row, row_c;
  bool row_ok;

  __device__ __forceinline__ GenRow() {
    const uint32_t tid = threadIdx.x;
    lane = BLOCK ? tid : (tid & (L - 1u));
    row = BLOCK ? blockIdx.x : blockIdx.x * ROWS_PER_WG + tid / L;
    row_ok = FULL_ROWS || row < ROWS;
    row_c = FULL_ROWS ? row : min(row, ROWS - 1u);
  }
  __device__ __forceinline__ bool valid(int k) const { return FULL_COLS || lane + k * LANES < NVEC; }
  __device__ __forceinline__ uint32_t vec_at(int k) const { return FULL_COLS ? lane + k * LANES : min(lane + k * LANES, NVEC - 1u); }

  // VEC elements of storage type T are W 128-bit words
  template <typename T>
  struct Raw {
    static constexpr int W = VEC * (int)sizeof(T) / 16;
    u32x4 w[K][W];
  };

  // the lane's K vectors of row `at_row` of a [.., COLS] tensor; STREAM: read once, bypass the caches' keep policy
  template <typename T, bool STREAM>
  __device__ __forceinline__ Raw<T> load(const void* p, size_t at_row) const {
    Raw<T> r;
    const T* base = static_cast<const T*>(p) + at_row * COLS;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const T* src = base + (size_t)vec_at(k) * VEC;
#pragma unroll
      for (int h = 0; h < Raw<T>::W; ++h) {
        const T* q = src + h * (16 / (int)sizeof(T));
        r.w[k][h] = STREAM ? load_raw_nt(q) : load_raw(q);
      }
    }
    return r;
  }

  template <typename T>
  __device__ __forceinline__ void unpack_to(const Raw<T>& r, float (&v)[KV]) const {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      if constexpr (Raw<T>::W == 1) {
        float part[VEC];
        unpack(r.w[k][0], part, (const T*)nullptr);
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[k * VEC + e] = part[e];
      } else {   // float32 under an 8-element step: two words
#pragma unroll
        for (int h = 0; h < Raw<T>::W; ++h) {
          float part[4];
          unpack(r.w[k][h], part, (const float*)nullptr);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[k * VEC + 4 * h + e] = part[e];
        }
      }
    }
  }

  template <typename TO>
  __device__ __forceinline__ void store(void* p, const float (&v)[KV]) const { store_at<TO>(p, (size_t)row, v); }

  // the row's values to row `at_row` of the output (its own row, or the place a folded transpose gives it)
  template <typename TO>
  __device__ __forceinline__ void store_at(void* p, size_t at_row, const float (&v)[KV]) const {
    TO* base = static_cast<TO*>(p) + at_row * COLS;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      float part[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) part[e] = v[k * VEC + e];
      if (row_ok && valid(k)) StoreN<TO, VEC>::run(base + (size_t)(lane + k * LANES) * VEC, part);
    }
  }

  template <typename TO>
  __device__ __forceinline__ void store_scalar(void* p, float v) const {
    if (row_ok && lane == 0) store1(static_cast<TO*>(p) + row, v);
  }

  // all-reduce over the row: every lane of the row ends with the same value.  SQUARE: of the squared
  // elements.  slot: 4 floats of LDS private to this reduction (BLOCK only).
  template <typename OP, bool IS_MAX, bool SQUARE>
  __device__ __forceinline__ float reduce(const float (&v)[KV], float* slot) const {
    // the lane's own elements are combined pairwise (a tree, not a chain): log2(KV) dependent steps instead of
    // KV, and a float32 sum whose rounding error grows with the depth of the tree
    float t[KV];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const bool ok = valid(k);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float x = SQUARE ? v[k * VEC + e] * v[k * VEC + e] : v[k * VEC + e];
        t[k * VEC + e] = FULL_COLS ? x : (ok ? x : (IS_MAX ? -__builtin_huge_valf() : 0.0f));
      }
    }
#pragma unroll
    for (int n = KV; n > 1; n = (n + 1) / 2) {
#pragma unroll
      for (int i = 0; i < n / 2; ++i) t[i] = OP::apply(t[2 * i], t[2 * i + 1]);
      if (n & 1) t[n / 2] = t[n - 1];
    }
    const float r = t[0];
    if constexpr (BLOCK) return block_allreduce<OP>(r, slot, 4);
    else return group_allreduce<OP>(r, (int)L);
  }
};

template <int DT> __device__ __forceinline__ float gen_round(float v) { return v; }
template <> __device__ __forceinline__ float gen_round<1>(float v) { return (float)(_Float16)v; }
template <> __device__ __forceinline__ float gen_round<2>(float v) { return bf16_bits_to_f32(pack_bf16(v, 0.0f) & 0xFFFFu); }

}  // namespace fsk
