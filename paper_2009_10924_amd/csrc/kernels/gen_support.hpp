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
  const void* full[8];
  const void* col[8];
  const void* rscal[8];
  void* out[8];
  void* rout[8];
  void* ws;   // partial column sums, one row per workgroup (patterns with column sums), else null
};

// Compile-time switches handed to generic lambdas of a generated kernel (`if constexpr (decltype(tag)::value)`).
struct Yes { static constexpr bool value = true; };
struct No { static constexpr bool value = false; };

// value of `v` in lane (own lane ^ mask) of the wavefront
__device__ __forceinline__ float xor_lane(float v, uint32_t mask) {
  const int addr = (int)(((threadIdx.x ^ mask) & 63u) << 2);
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr, __builtin_bit_cast(int, v)));
}

// One step of one lane in storage form: VEC elements of 2 or 4 bytes are 2, 4, 8, 16 or 32 bytes.  VEC is 8 or 4
// where the row length allows 128-bit (or, for 16-bit elements under VEC = 4, 64-bit) accesses, and 1 for rows
// whose length is not a multiple of 4 elements: every access is then a single element, still contiguous over
// the lanes of a row.
template <int BYTES> struct StepBits;
template <> struct StepBits<32> {
  u32x4 lo, hi;
  template <bool STREAM, typename T>
  __device__ __forceinline__ static StepBits load(const T* p) {
    StepBits r;
    const u32x4* q = reinterpret_cast<const u32x4*>(p);
    r.lo = STREAM ? __builtin_nontemporal_load(q) : q[0];
    r.hi = STREAM ? __builtin_nontemporal_load(q + 1) : q[1];
    return r;
  }
};
template <> struct StepBits<16> {
  u32x4 w;
  template <bool STREAM, typename T>
  __device__ __forceinline__ static StepBits load(const T* p) {
    StepBits r;
    r.w = STREAM ? load_raw_nt(p) : load_raw(p);
    return r;
  }
};
template <> struct StepBits<8> {
  u32x2 w;
  template <bool STREAM, typename T>
  __device__ __forceinline__ static StepBits load(const T* p) {
    StepBits r;
    const u32x2* q = reinterpret_cast<const u32x2*>(p);
    r.w = STREAM ? __builtin_nontemporal_load(q) : *q;
    return r;
  }
};
template <> struct StepBits<4> {
  uint32_t w;
  template <bool STREAM, typename T>
  __device__ __forceinline__ static StepBits load(const T* p) {
    StepBits r;
    const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
    r.w = STREAM ? __builtin_nontemporal_load(q) : *q;
    return r;
  }
};
template <> struct StepBits<2> {
  uint16_t w;
  template <bool STREAM, typename T>
  __device__ __forceinline__ static StepBits load(const T* p) {
    StepBits r;
    const uint16_t* q = reinterpret_cast<const uint16_t*>(p);
    r.w = STREAM ? __builtin_nontemporal_load(q) : *q;
    return r;
  }
};
// Registers that hold a step in storage form across several passes: after this the compiler no longer knows what is
// in them, so it cannot carry the unpacked float32 form (twice the registers of a 16-bit step) from one pass to the
// next instead.  No instruction is emitted.
__device__ __forceinline__ void forget_contents(StepBits<32>& s) { asm volatile("" : "+v"(s.lo), "+v"(s.hi)); }
__device__ __forceinline__ void forget_contents(StepBits<16>& s) { asm volatile("" : "+v"(s.w)); }
__device__ __forceinline__ void forget_contents(StepBits<8>& s) { asm volatile("" : "+v"(s.w)); }
__device__ __forceinline__ void forget_contents(StepBits<4>& s) { asm volatile("" : "+v"(s.w)); }
__device__ __forceinline__ void forget_contents(StepBits<2>& s) {
  uint32_t t = s.w;
  asm volatile("" : "+v"(t));
  s.w = (uint16_t)t;
}

__device__ __forceinline__ void unpack_step(const StepBits<32>& r, float (&v)[8], const float*) {
  float a[4], b[4];
  unpack(r.lo, a, (const float*)nullptr);
  unpack(r.hi, b, (const float*)nullptr);
#pragma unroll
  for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
}
__device__ __forceinline__ void unpack_step(const StepBits<16>& r, float (&v)[4], const float*) { unpack(r.w, v, (const float*)nullptr); }
template <typename T>
__device__ __forceinline__ void unpack_step(const StepBits<16>& r, float (&v)[8], const T*) { unpack(r.w, v, (const T*)nullptr); }
__device__ __forceinline__ void unpack_step(const StepBits<8>& r, float (&v)[4], const bf16_t*) {
  v[0] = __builtin_bit_cast(float, r.w.x << 16); v[1] = __builtin_bit_cast(float, r.w.x & 0xFFFF0000u);
  v[2] = __builtin_bit_cast(float, r.w.y << 16); v[3] = __builtin_bit_cast(float, r.w.y & 0xFFFF0000u);
}
__device__ __forceinline__ void unpack_step(const StepBits<8>& r, float (&v)[4], const f16_t*) {
  unpack_f16(r.w.x, v[0], v[1]);
  unpack_f16(r.w.y, v[2], v[3]);
}
__device__ __forceinline__ void unpack_step(const StepBits<4>& r, float (&v)[1], const float*) { v[0] = __builtin_bit_cast(float, r.w); }
__device__ __forceinline__ void unpack_step(const StepBits<2>& r, float (&v)[1], const bf16_t*) { v[0] = bf16_bits_to_f32(r.w); }
__device__ __forceinline__ void unpack_step(const StepBits<2>& r, float (&v)[1], const f16_t*) {
  v[0] = (float)__builtin_bit_cast(_Float16, r.w);
}

// ROWS x COLS row space; VEC elements per lane and step; K steps per lane; L lanes per row: a lane group of one
// wavefront in a 256-thread workgroup, or, when BLOCK, the whole workgroup of L = 256, 512 or 1024 threads.
// R: rows each lane group works through, one after the other (the kernel body runs R times with virtual
// workgroup indices it * gridDim.x + blockIdx.x, so that at any moment the resident workgroups sweep one band of rows).
// ROW_STRIDE > COLS: the pattern's rows are ROW_STRIDE elements long and the kernel works on column tiles of COLS
// elements (patterns without row reductions only: nothing ties the tiles of a row together); `tile` picks the tile.
template <uint32_t ROWS, uint32_t COLS, int VEC, int K, uint32_t L, bool BLOCK, uint32_t R = 1, uint32_t ROW_STRIDE = COLS>
struct GenRow {
  static constexpr uint32_t NVEC = COLS / VEC;
  static constexpr uint32_t LANES = L;
  static constexpr uint32_t ROWS_PER_WG = BLOCK ? 1u : 256u / L;
  // the row fills its lanes / the rows fill the workgroups: no clamp, no padding test
  static constexpr bool FULL_COLS = NVEC == LANES * K;
  static constexpr bool FULL_ROWS = ROWS % (ROWS_PER_WG * R) == 0;
  static constexpr int KV = K * VEC;
  static constexpr uint32_t PADDED_COLS = LANES * K * VEC;   // columns the lanes of a row cover, padding included

  uint32_t lane, row, row_c, col0;
  bool row_ok;

  __device__ __forceinline__ explicit GenRow(uint32_t vblock, uint32_t tile = 0) {
    const uint32_t tid = threadIdx.x;
    col0 = tile * COLS;
    lane = BLOCK ? tid : (tid & (L - 1u));
    row = BLOCK ? vblock : vblock * ROWS_PER_WG + tid / L;
    row_ok = FULL_ROWS || row < ROWS;
    row_c = FULL_ROWS ? row : min(row, ROWS - 1u);
  }
  // a chunk of a long row: COLS columns from column `first_col` on (the row itself is ROW_STRIDE elements long)
  __device__ __forceinline__ GenRow(uint32_t vblock, uint32_t tile, uint32_t first_col) : GenRow(vblock, tile) { col0 = first_col; }
  __device__ __forceinline__ bool valid(int k) const { return FULL_COLS || lane + k * LANES < NVEC; }
  __device__ __forceinline__ uint32_t vec_at(int k) const { return FULL_COLS ? lane + k * LANES : min(lane + k * LANES, NVEC - 1u); }

  // the lane's K steps of row `at_row` of a [.., COLS] tensor, in storage form; STREAM: read once, so the loads
  // carry the streaming hint and do not displace the operands that every row re-reads from cache
  template <typename T>
  struct Raw {
    StepBits<VEC * (int)sizeof(T)> w[K];
    __device__ __forceinline__ void forget_contents() {
#pragma unroll
      for (int k = 0; k < K; ++k) fsk::forget_contents(w[k]);
    }
  };
  template <typename T, bool STREAM>
  __device__ __forceinline__ Raw<T> load(const void* p, size_t at_row) const {
    Raw<T> r;
    const T* base = static_cast<const T*>(p) + at_row * ROW_STRIDE + col0;
#pragma unroll
    for (int k = 0; k < K; ++k) r.w[k] = StepBits<VEC * (int)sizeof(T)>::template load<STREAM>(base + (size_t)vec_at(k) * VEC);
    return r;
  }

  template <typename T>
  __device__ __forceinline__ void unpack_to(const Raw<T>& r, float (&v)[KV]) const {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      float part[VEC];
      unpack_step(r.w[k], part, (const T*)nullptr);
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[k * VEC + e] = part[e];
    }
  }

  template <typename TO>
  __device__ __forceinline__ void store(void* p, const float (&v)[KV]) const { store_at<TO>(p, (size_t)row, v); }

  // the row's values to row `at_row` of the output (its own row, or the place a folded transpose gives it)
  template <typename TO>
  __device__ __forceinline__ void store_at(void* p, size_t at_row, const float (&v)[KV]) const {
    TO* base = static_cast<TO*>(p) + at_row * ROW_STRIDE + col0;
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
  // elements.  slot: one float per wavefront of the workgroup, LDS private to this reduction (BLOCK only).
  template <typename OP, bool IS_MAX, bool SQUARE>
  __device__ __forceinline__ float reduce(const float (&v)[KV], float* slot) const {
    return finish<OP>(partial<OP, IS_MAX, SQUARE>(v), slot);
  }
  // the two halves of reduce(): the lane's own elements folded to one value (rows worked through in chunks fold
  // their chunks' values lane by lane first), and the all-reduce of the lanes' values over the row
  template <typename OP, bool IS_MAX, bool SQUARE>
  __device__ __forceinline__ float partial(const float (&v)[KV]) const {
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
    return t[0];
  }
  template <typename OP>
  __device__ __forceinline__ static float finish(float r, float* slot) {
    if constexpr (BLOCK) return block_allreduce<OP>(r, slot, (int)(L / 64u));
    else return group_allreduce<OP>(r, (int)L);
  }

  // ---- column sums over all rows (lane-group rows only) ----------------------------------------------------
  // the row's values join the lane's running sums; padding lanes and rows beyond the last add nothing
  __device__ __forceinline__ void colsum_add(const float (&v)[KV], float (&sum)[KV]) const {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const bool ok = row_ok && valid(k);
#pragma unroll
      for (int e = 0; e < VEC; ++e) sum[k * VEC + e] += ok ? v[k * VEC + e] : 0.0f;
    }
  }
  // Lane-group rows: the workgroup's lane groups hold sums of the same columns: first the groups of a wavefront are folded lane to
  // lane (lane ^ L, lane ^ 2L, ...: every lane ends with the wavefront's sum), then the four wavefronts through
  // `lds` (4 * PADDED_COLS floats, used by this sum only), and one row of COLS partial sums goes to `dst`.  Fixed
  // order throughout, so the result is the same from run to run.
  __device__ __forceinline__ static void colsum_flush(const float (&sum)[KV], float* lds, float* dst) {
    if constexpr (BLOCK) {
      // a workgroup per row: every lane owns its columns alone, the sums over the workgroup's rows are complete
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const uint32_t at = (threadIdx.x + k * L) * VEC;
        if (FULL_COLS || at < COLS) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) dst[at + e] = sum[k * VEC + e];
        }
      }
      return;
    }
    float v[KV];
#pragma unroll
    for (int j = 0; j < KV; ++j) v[j] = sum[j];
#pragma unroll
    for (uint32_t s = L; s < 64u; s <<= 1) {
#pragma unroll
      for (int j = 0; j < KV; ++j) v[j] += xor_lane(v[j], s);
    }
    const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & (L - 1u);
    if ((tid & 63u) < L) {
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int e = 0; e < VEC; ++e) lds[wave * PADDED_COLS + (lane + k * L) * VEC + e] = v[k * VEC + e];
    }
    __syncthreads();
    for (uint32_t c = tid; c < COLS; c += 256u)
      dst[c] = ((lds[c] + lds[PADDED_COLS + c]) + lds[2u * PADDED_COLS + c]) + lds[3u * PADDED_COLS + c];
  }
};

// A mid-pattern `convert`: the float32 value rounded to the storage dtype (nearest even) and widened again.  The value
// is pinned in a register first (an empty asm the compiler cannot see through): otherwise the compiler may fuse the
// multiplication that produced it with the conversion into one mixed-precision instruction (v_fma_mixlo_f16), which
// rounds the exact product once -- while another use of the same value (the store) rounds the float32 product.  The
// two differ by one 16-bit ulp where the float32 product is a tie, and a column sum of the rounded values would no
// longer be the sum of what is stored.
template <int DT> __device__ __forceinline__ float gen_round(float v) { return v; }
template <> __device__ __forceinline__ float gen_round<1>(float v) {
  asm volatile("" : "+v"(v));
  return (float)(_Float16)v;
}
template <> __device__ __forceinline__ float gen_round<2>(float v) {
  asm volatile("" : "+v"(v));
  return bf16_bits_to_f32(pack_bf16(v, 0.0f) & 0xFFFFu);
}

}  // namespace fsk
