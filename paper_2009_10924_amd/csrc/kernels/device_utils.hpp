// Device-side helpers for gfx950: 128-bit typed loads/stores that widen to float32,
// round-to-nearest-even narrowing, and wave64 cross-lane reductions.
#pragma once
#ifndef __HIPCC_RTC__
#include <hip/hip_runtime.h>
#include <stdint.h>
#else
// run-time compilation: the HIP device declarations are built in, the C headers are not there
typedef unsigned int uint32_t;
typedef unsigned short uint16_t;
#endif

namespace fsk {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

struct bf16_t { uint16_t bits; };   // storage tag types; arithmetic is always float32
typedef _Float16 f16_t;

constexpr int kWave = 64;

// ---- element traits: VEC = elements in one 128-bit access --------------------
template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int VEC = 4; };
template <> struct Elem<f16_t> { static constexpr int VEC = 8; };
template <> struct Elem<bf16_t> { static constexpr int VEC = 8; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __builtin_bit_cast(float, b << 16); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 r = __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32: round to nearest even
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
  f16x2 r = {(_Float16)lo, (_Float16)hi};          // v_cvt_f16_f32: round to nearest even
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ void unpack_f16(uint32_t w, float& lo, float& hi) {
  f16x2 h = __builtin_bit_cast(f16x2, w);
  lo = (float)h.x;
  hi = (float)h.y;
}

// ---- scalar element access ---------------------------------------------------
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const f16_t* p) { return (float)*p; }
__device__ __forceinline__ float load1(const bf16_t* p) { return bf16_bits_to_f32(p->bits); }
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(f16_t* p, float v) { *p = (_Float16)v; }
__device__ __forceinline__ void store1(bf16_t* p, float v) {
  p->bits = __builtin_bit_cast(uint16_t, (__bf16)v);
}

// ---- 128-bit vector access: VEC elements <-> float[VEC] -----------------------
__device__ __forceinline__ void load_vec(const float* p, float (&v)[4]) {
  f32x4 t = *reinterpret_cast<const f32x4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load_vec(const bf16_t* p, float (&v)[8]) {
  u32x4 t = *reinterpret_cast<const u32x4*>(p);
  v[0] = __builtin_bit_cast(float, t.x << 16); v[1] = __builtin_bit_cast(float, t.x & 0xFFFF0000u);
  v[2] = __builtin_bit_cast(float, t.y << 16); v[3] = __builtin_bit_cast(float, t.y & 0xFFFF0000u);
  v[4] = __builtin_bit_cast(float, t.z << 16); v[5] = __builtin_bit_cast(float, t.z & 0xFFFF0000u);
  v[6] = __builtin_bit_cast(float, t.w << 16); v[7] = __builtin_bit_cast(float, t.w & 0xFFFF0000u);
}
__device__ __forceinline__ void load_vec(const f16_t* p, float (&v)[8]) {
  u32x4 t = *reinterpret_cast<const u32x4*>(p);
  unpack_f16(t.x, v[0], v[1]); unpack_f16(t.y, v[2], v[3]);
  unpack_f16(t.z, v[4], v[5]); unpack_f16(t.w, v[6], v[7]);
}
__device__ __forceinline__ void store_vec(float* p, const float (&v)[4]) {
  f32x4 t = {v[0], v[1], v[2], v[3]};
  *reinterpret_cast<f32x4*>(p) = t;
}
__device__ __forceinline__ void store_vec(bf16_t* p, const float (&v)[8]) {
  u32x4 t = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
  *reinterpret_cast<u32x4*>(p) = t;
}
__device__ __forceinline__ void store_vec(f16_t* p, const float (&v)[8]) {
  u32x4 t = {pack_f16(v[0], v[1]), pack_f16(v[2], v[3]), pack_f16(v[4], v[5]), pack_f16(v[6], v[7])};
  *reinterpret_cast<u32x4*>(p) = t;
}
// ---- raw 128-bit access with a streaming (non-temporal) hint ------------------------
// Inputs read once and outputs written once should not displace the small operands
// (bias, gamma, mask) that every row re-reads from cache.  A kernel first issues all
// its raw loads, then unpacks: the loads stay independent of any arithmetic and of
// each other, so they are all in flight together.
template <typename T>
__device__ __forceinline__ u32x4 load_raw_nt(const T* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
template <typename T>
__device__ __forceinline__ u32x4 load_raw(const T* p) {
  return *reinterpret_cast<const u32x4*>(p);
}
__device__ __forceinline__ void unpack(u32x4 t, float (&v)[4], const float*) {
  // the whole vector is re-typed first: bit-casting a single vector element (an lvalue
  // like t.y) is miscompiled by this toolchain into a read of element 0
  const f32x4 f = __builtin_bit_cast(f32x4, t);
  v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
}
__device__ __forceinline__ void unpack(u32x4 t, float (&v)[8], const bf16_t*) {
  v[0] = __builtin_bit_cast(float, t.x << 16); v[1] = __builtin_bit_cast(float, t.x & 0xFFFF0000u);
  v[2] = __builtin_bit_cast(float, t.y << 16); v[3] = __builtin_bit_cast(float, t.y & 0xFFFF0000u);
  v[4] = __builtin_bit_cast(float, t.z << 16); v[5] = __builtin_bit_cast(float, t.z & 0xFFFF0000u);
  v[6] = __builtin_bit_cast(float, t.w << 16); v[7] = __builtin_bit_cast(float, t.w & 0xFFFF0000u);
}
__device__ __forceinline__ void unpack(u32x4 t, float (&v)[8], const f16_t*) {
  unpack_f16(t.x, v[0], v[1]); unpack_f16(t.y, v[2], v[3]);
  unpack_f16(t.z, v[4], v[5]); unpack_f16(t.w, v[6], v[7]);
}
__device__ __forceinline__ void store_vec_nt(float* p, const float (&v)[4]) {
  f32x4 t = {v[0], v[1], v[2], v[3]};
  __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(p));
}
__device__ __forceinline__ void store_vec_nt(bf16_t* p, const float (&v)[8]) {
  u32x4 t = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void store_vec_nt(f16_t* p, const float (&v)[8]) {
  u32x4 t = {pack_f16(v[0], v[1]), pack_f16(v[2], v[3]), pack_f16(v[4], v[5]), pack_f16(v[6], v[7])};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void store_vec4_nt(float* p, const float (&v)[4]) { store_vec_nt(p, v); }
__device__ __forceinline__ void store_vec4_nt(bf16_t* p, const float (&v)[4]) {
  u32x2 t = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
}
__device__ __forceinline__ void store_vec4_nt(f16_t* p, const float (&v)[4]) {
  u32x2 t = {pack_f16(v[0], v[1]), pack_f16(v[2], v[3])};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
}

// 4-element (64-bit) access for 16-bit types, used when a float32 vector of 4 pairs with them.
__device__ __forceinline__ void load_vec4(const float* p, float (&v)[4]) { load_vec(p, v); }
__device__ __forceinline__ void load_vec4(const bf16_t* p, float (&v)[4]) {
  u32x2 t = *reinterpret_cast<const u32x2*>(p);
  v[0] = __builtin_bit_cast(float, t.x << 16); v[1] = __builtin_bit_cast(float, t.x & 0xFFFF0000u);
  v[2] = __builtin_bit_cast(float, t.y << 16); v[3] = __builtin_bit_cast(float, t.y & 0xFFFF0000u);
}
__device__ __forceinline__ void load_vec4(const f16_t* p, float (&v)[4]) {
  u32x2 t = *reinterpret_cast<const u32x2*>(p);
  unpack_f16(t.x, v[0], v[1]); unpack_f16(t.y, v[2], v[3]);
}
__device__ __forceinline__ void store_vec4(float* p, const float (&v)[4]) { store_vec(p, v); }
__device__ __forceinline__ void store_vec4(bf16_t* p, const float (&v)[4]) {
  u32x2 t = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
  *reinterpret_cast<u32x2*>(p) = t;
}
__device__ __forceinline__ void store_vec4(f16_t* p, const float (&v)[4]) {
  u32x2 t = {pack_f16(v[0], v[1]), pack_f16(v[2], v[3])};
  *reinterpret_cast<u32x2*>(p) = t;
}

// Stores VEC(TI) float32 values as TO: a full 128-bit access when the two types are equally
// wide, a 64-bit one when float32 rows are stored as a 16-bit type.
template <typename TO, int N> struct StoreN;
template <typename TO> struct StoreN<TO, 1> {   // rows whose length allows no wider access: one element
  __device__ __forceinline__ static void run(TO* p, const float (&v)[1]) { store1(p, v[0]); }
};
template <typename TO> struct StoreN<TO, 4> {
  __device__ __forceinline__ static void run(TO* p, const float (&v)[4]) { store_vec4_nt(p, v); }
};
template <> struct StoreN<float, 8> {
  __device__ __forceinline__ static void run(float* p, const float (&v)[8]) {
    float a[4] = {v[0], v[1], v[2], v[3]}, b[4] = {v[4], v[5], v[6], v[7]};
    store_vec_nt(p, a);
    store_vec_nt(p + 4, b);
  }
};
template <> struct StoreN<f16_t, 8> {
  __device__ __forceinline__ static void run(f16_t* p, const float (&v)[8]) { store_vec_nt(p, v); }
};
template <> struct StoreN<bf16_t, 8> {
  __device__ __forceinline__ static void run(bf16_t* p, const float (&v)[8]) { store_vec_nt(p, v); }
};

// ---- division by a run-time constant (see fs::FastDiv) -------------------------------
template <typename FD>
__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FD& f) {
  return f.d == 1 ? n : (__umulhi(n, f.m) >> f.s);
}

// ---- math ---------------------------------------------------------------------
constexpr float kLog2e = 1.4426950408889634f;
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_rsqrt(float x) { return __builtin_amdgcn_rsqf(x); }
// 1 / (1 + exp(-x)); saturates to 0 and 1 by itself (exp2 overflows to +inf, whose reciprocal is 0)
__device__ __forceinline__ float fast_sigmoid(float x) { return fast_rcp(1.0f + __builtin_amdgcn_exp2f(-kLog2e * x)); }
// the compiler's own expansions (no library call): accurate to about one unit in the last place over the whole range
__device__ __forceinline__ float full_log(float x) { return __builtin_logf(x); }
__device__ __forceinline__ float full_sqrt(float x) { return __builtin_sqrtf(x); }

// tanh without the library routine's range reduction: 1 - 2/(1 + exp(2x)) away from zero (saturates to +-1 by
// itself), the odd Taylor polynomial up to x^7 below |x| = 0.25 where the first form cancels.  Relative error
// below 1e-6 over the whole range.
__device__ __forceinline__ float fast_tanh(float x) {
  const float x2 = x * x;
  const float small = x * __builtin_fmaf(x2, __builtin_fmaf(x2, __builtin_fmaf(x2, -17.0f / 315.0f, 2.0f / 15.0f), -1.0f / 3.0f), 1.0f);
  const float big = 1.0f - 2.0f * fast_rcp(1.0f + __builtin_amdgcn_exp2f(2.0f * kLog2e * x));
  return fabsf(x) < 0.25f ? small : big;
}

// tanh-GELU through the logistic form: gelu(z) = z * s, s = 1/(1+exp(-2u)),
// u = sqrt(2/pi) (z + 0.044715 z^3).  Same function as z/2 (1+tanh u) in exact
// arithmetic, without the cancellation of 1+tanh(u) for z << 0.
__device__ __forceinline__ void gelu_parts(float z, float& s, float& dcoef) {
  constexpr float k2c = 2.0f * 0.7978845608028654f;          // 2 sqrt(2/pi)
  const float z2 = z * z;
  const float w = k2c * z * __builtin_fmaf(0.044715f, z2, 1.0f);   // 2u
  s = fast_rcp(1.0f + __builtin_amdgcn_exp2f(-kLog2e * w));
  dcoef = k2c * __builtin_fmaf(3.0f * 0.044715f, z2, 1.0f);        // d(2u)/dz
}
__device__ __forceinline__ float gelu_fwd(float z) {
  float s, d;
  gelu_parts(z, s, d);
  return z * s;
}
__device__ __forceinline__ float gelu_grad(float z) {
  float s, d;
  gelu_parts(z, s, d);
  return __builtin_fmaf(z * s * (1.0f - s), d, s);
}

// ---- wave64 cross-lane all-reduce over aligned groups of L lanes (L power of two) ----
// Steps inside a 16-lane DPP row use DPP operand modifiers (no LDS traffic); the
// 32- and 64-lane steps use ds_bpermute.  Every lane of the group ends with the
// same bits: each step combines two values that both sides hold, with a
// commutative op.
struct OpSum { __device__ __forceinline__ static float apply(float a, float b) { return a + b; } };
struct OpMax { __device__ __forceinline__ static float apply(float a, float b) { return fmaxf(a, b); } };

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

__device__ __forceinline__ float read_lane(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// Branch-free on purpose: `lanes` is wave-uniform, each step is computed and then kept
// or dropped by a select.  Without branches a kernel's loads, reductions and stores
// stay in one basic block, so the scheduler keeps early loads early instead of sinking
// them next to their first use behind the reduction.
template <typename OP>
__device__ __forceinline__ float group_allreduce(float v, int lanes) {
  float t;
  t = OP::apply(v, dpp_move<0xB1>(v));  v = lanes > 1 ? t : v;   // quad_perm [1,0,3,2] : lane ^ 1
  t = OP::apply(v, dpp_move<0x4E>(v));  v = lanes > 2 ? t : v;   // quad_perm [2,3,0,1] : lane ^ 2
  t = OP::apply(v, dpp_move<0x141>(v)); v = lanes > 4 ? t : v;   // row_half_mirror     : other quad of the 8
  t = OP::apply(v, dpp_move<0x140>(v)); v = lanes > 8 ? t : v;   // row_mirror          : other half of the 16
  // every 16-lane row now holds its own total in all lanes: rows are combined through
  // scalar registers (v_readlane), which costs no LDS-crossbar round trip.
  const float lo = OP::apply(read_lane(v, 0), read_lane(v, 16));
  const float hi = OP::apply(read_lane(v, 32), read_lane(v, 48));
  const float half = (threadIdx.x & 32u) ? hi : lo;
  const float full = OP::apply(lo, hi);
  return lanes > 32 ? full : (lanes > 16 ? half : v);
}

// Workgroup all-reduce through LDS (block composition): each wave reduces, lane 0
// of each wave parks its value, after the barrier every thread folds the parked
// values in wave order.  `slot` must hold blockDim.x/64 floats; the caller owns
// reuse of `slot` (a barrier separates two uses).
template <typename OP>
__device__ __forceinline__ float block_allreduce(float v, float* slot, int n_waves) {
  v = group_allreduce<OP>(v, kWave);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) slot[wave] = v;
  __syncthreads();
  float r = slot[0];
  for (int w = 1; w < n_waves; ++w) r = OP::apply(r, slot[w]);
  return r;
}

}  // namespace fsk
