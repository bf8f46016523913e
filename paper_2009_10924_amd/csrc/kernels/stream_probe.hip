// Streaming probes: what the memory system gives a kernel that does nothing but move data,
// for a given mix of read and write streams.  A stitched kernel is reported beside the probe
// with its own mix (the paper's Section 2.2: off-chip traffic is what memory-intensive ops
// spend their time on, so the traffic-only kernel is the bound to compare with).
// One-shot shape, like the stitched row kernels: a lane takes K 128-bit vectors of every
// stream, all loads are issued before anything else, stores carry the streaming hint.
#include <hip/hip_runtime.h>

#include "../fs_internal.hpp"
#include "device_utils.hpp"

namespace fsk {

template <int R, int W, int K>
__global__ void __launch_bounds__(256) k_stream_probe(const u32x4* __restrict__ src, u32x4* __restrict__ dst, uint32_t n_vec, uint32_t pitch_vec) {
  const uint32_t base = blockIdx.x * (256u * K) + threadIdx.x;
  u32x4 t[R > 0 ? R : 1][K];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int k = 0; k < K; ++k)
      t[r][k] = __builtin_nontemporal_load(src + (size_t)r * pitch_vec + min(base + k * 256u, n_vec - 1u));   // clamped, not branched
  u32x4 v[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const uint32_t i = base + k * 256u;
    v[k] = u32x4{i, i, i, i};
#pragma unroll
    for (int r = 0; r < R; ++r) v[k] ^= t[r][k];
  }
  if constexpr (W == 0) {
    // keeps the loads alive: the buffers never hold this pattern
#pragma unroll
    for (int k = 0; k < K; ++k)
      if (v[k].x == 0x7fc12345u && v[k].y == 0x13572468u && v[k].z == 0x0badf00du) dst[0] = v[k];
  } else {
#pragma unroll
    for (int w = 0; w < W; ++w)
#pragma unroll
      for (int k = 0; k < K; ++k)
        if (base + k * 256u < n_vec) __builtin_nontemporal_store(v[k], dst + (size_t)w * pitch_vec + base + k * 256u);
  }
}

template <int R, int W>
const void* probe_k(int k) {
  switch (k) {
    case 1: return (const void*)k_stream_probe<R, W, 1>;
    case 2: return (const void*)k_stream_probe<R, W, 2>;
    case 4: return (const void*)k_stream_probe<R, W, 4>;
    default: return nullptr;
  }
}
template <int R>
const void* probe_w(int w, int k) {
  switch (w) {
    case 0: return R == 0 ? nullptr : probe_k<R, 0>(k);
    case 1: return probe_k<R, 1>(k);
    case 2: return probe_k<R, 2>(k);
    default: return nullptr;
  }
}
const void* probe_symbol(int r, int w, int k) {
  switch (r) {
    case 0: return probe_w<0>(w, k);
    case 1: return probe_w<1>(w, k);
    case 2: return probe_w<2>(w, k);
    case 3: return probe_w<3>(w, k);
    case 4: return probe_w<4>(w, k);
    default: return nullptr;
  }
}

}  // namespace fsk

extern "C" fs_status fs_stream_probe(void* dst, const void* src, size_t stream_bytes, size_t stream_pitch_bytes, int32_t reads,
                                     int32_t writes, int32_t vecs_per_lane, void* hip_stream) try {
  fs::clear_error();
  if (!dst || (reads > 0 && !src)) return fs::fail(FS_ERR_INVALID_ARG, "fs_stream_probe: null pointer");
  const void* sym = fsk::probe_symbol(reads, writes, vecs_per_lane);
  if (!sym)
    return fs::fail(FS_ERR_INVALID_ARG, "fs_stream_probe: reads 0..4, writes 0..2 (not both 0), vecs_per_lane 1, 2 or 4; got %d, %d, %d", reads, writes,
                    vecs_per_lane);
  if (stream_pitch_bytes == 0) stream_pitch_bytes = stream_bytes;
  if (((uintptr_t)dst | (uintptr_t)src | stream_bytes | stream_pitch_bytes) & 15u)
    return fs::fail(FS_ERR_ALIGN, "fs_stream_probe: pointers, size and pitch must be multiples of 16");
  if (stream_pitch_bytes < stream_bytes) return fs::fail(FS_ERR_SHAPE, "fs_stream_probe: the pitch is smaller than a stream");
  if (stream_bytes == 0) return FS_OK;
  if (stream_pitch_bytes / 16 >= (size_t(1) << 31)) return fs::fail(FS_ERR_SHAPE, "fs_stream_probe: too large");
  uint32_t n_vec = (uint32_t)(stream_bytes / 16), pitch_vec = (uint32_t)(stream_pitch_bytes / 16);
  const uint32_t per_block = 256u * (uint32_t)vecs_per_lane;
  void* argv[4] = {&src, &dst, &n_vec, &pitch_vec};
  const hipError_t e = hipLaunchKernel(sym, dim3((n_vec + per_block - 1) / per_block), dim3(256), argv, 0, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fs::fail(FS_ERR_HIP, "fs_stream_probe: %s", hipGetErrorString(e));
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_stream_probe");
}
