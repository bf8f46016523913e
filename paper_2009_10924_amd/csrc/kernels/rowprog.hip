// Interpreted row program: the generic code path for fusion patterns no hand-written
// kernel family covers (paper Section 4: any pattern of memory-intensive ops whose reuse
// stays inside a warp or a block is one kernel).  A pattern of element-wise ops,
// broadcasts and last-axis reductions over one [rows, cols] space is compiled on the host
// into a short instruction list; this kernel executes it with
//   * a row per lane group of one wavefront (warp composition) or per workgroup (block
//     composition), exactly like the hand-written row kernels,
//   * every global load issued before the first instruction runs, each input read once,
//   * column vectors in an LDS file shared by the workgroup; full-shaped values in THE
//     accumulator (VGPRs: every instruction reads and writes it) or a per-lane register file in LDS (a lane only ever touches its own
//     slots, so no barrier guards them); inputs are parked there by the prologue,
//   * per-row values (reduction results and what is computed from them) in a scalar
//     accumulator or a per-lane scalar file, identical in all lanes of the row,
//   * outputs written once, rounded at the store.
// The instruction walk is uniform over the workgroup: all control flow is scalar.
#include <hip/hip_runtime.h>

#include "kernel_table.hpp"
#include "row_skeleton.hpp"

namespace fsk {

typedef const ProgArgs __attribute__((address_space(4))) * ConstProgArgs;

__device__ __forceinline__ float round_through(float v, int dt) {
  if (dt == DT_F16) return (float)(_Float16)v;
  if (dt == DT_BF16) return bf16_bits_to_f32(pack_bf16(v, 0.0f) & 0xFFFFu);
  return v;
}

__device__ __forceinline__ float load_scalar_as(const void* p, size_t i, int dt) {
  if (dt == DT_F16) return load1(static_cast<const f16_t*>(p) + i);
  if (dt == DT_BF16) return load1(static_cast<const bf16_t*>(p) + i);
  return load1(static_cast<const float*>(p) + i);
}

__device__ __forceinline__ void store_scalar_as(void* p, size_t i, int dt, float v) {
  if (dt == DT_F16) store1(static_cast<f16_t*>(p) + i, v);
  else if (dt == DT_BF16) store1(static_cast<bf16_t*>(p) + i, v);
  else store1(static_cast<float*>(p) + i, v);
}

// a = the accumulator, b = the other operand
__device__ __forceinline__ float apply_op(int op, float a, float b, int aux) {
  switch (op) {
    case PO_ADD: return a + b;
    case PO_SUB: return a - b;
    case PO_RSUB: return b - a;
    case PO_MUL: return a * b;
    case PO_DIV: return a * fast_rcp(b);
    case PO_RDIV: return b * fast_rcp(a);
    case PO_MAX: return fmaxf(a, b);
    case PO_SQUARE: return a * a;
    case PO_EXP: return fast_exp(a);
    case PO_RSQRT: return fast_rsqrt(a);
    case PO_TANH: return fast_tanh(a);
    case PO_GELU: return gelu_fwd(a);
    case PO_GELU_GRAD: return gelu_grad(a);
    case PO_LOG: return full_log(a);
    case PO_SIGMOID: return fast_sigmoid(a);
    case PO_RELU: return fmaxf(a, 0.0f);
    case PO_ABS: return __builtin_fabsf(a);
    case PO_SQRT: return full_sqrt(a);
    case PO_CVT: return round_through(a, aux);
    default: return b;   // PO_LOAD
  }
}

// VEC elements of a row per lane and step (8 as soon as one vector input is 16-bit wide, so that the narrow
// inputs still move in 128-bit accesses; a float32 input then takes two).  NI: capacity for full-shaped inputs
// (sizes the prologue's load batch).
template <int VEC, int W>
struct RawVec {      // VEC elements in storage form: W 128-bit words
  u32x4 w[W];
};
template <int VEC>
__device__ __forceinline__ RawVec<VEC, VEC / 4> load_elems(const void* p, size_t at, int dt, bool streaming) {
  RawVec<VEC, VEC / 4> r;
#pragma unroll
  for (int h = 0; h < VEC / 4; ++h) r.w[h] = u32x4{0u, 0u, 0u, 0u};
  if (VEC == 4 || dt == DT_F32) {   // a vec-4 program has float32 vector inputs only: no test at run time
    const float* src = static_cast<const float*>(p) + at;
#pragma unroll
    for (int h = 0; h < VEC / 4; ++h) r.w[h] = streaming ? load_raw_nt(src + 4 * h) : load_raw(src + 4 * h);
  } else if (VEC == 8) {
    const uint16_t* src = static_cast<const uint16_t*>(p) + at;
    r.w[0] = streaming ? load_raw_nt(src) : load_raw(src);
  }
  return r;
}
template <int VEC>
__device__ __forceinline__ void unpack_elems(const RawVec<VEC, VEC / 4>& r, int dt, float (&v)[VEC]) {
  if (VEC == 4 || dt == DT_F32) {
#pragma unroll
    for (int h = 0; h < VEC / 4; ++h) {
      float part[4];
      unpack(r.w[h], part, (const float*)nullptr);
      v[4 * h] = part[0]; v[4 * h + 1] = part[1]; v[4 * h + 2] = part[2]; v[4 * h + 3] = part[3];
    }
  } else if constexpr (VEC == 8) {
    if (dt == DT_F16) unpack(r.w[0], v, (const f16_t*)nullptr);
    else unpack(r.w[0], v, (const bf16_t*)nullptr);
  }
}

template <int VEC, int K, int NI>
__global__ void __launch_bounds__(256) k_row_program(const ProgArgs args_in_kernarg) {
  constexpr int KV = K * VEC;     // floats a lane holds per full-shaped value
  constexpr int CH = KV / 4;      // 16-byte chunks of one register of one lane
  extern __shared__ f32x4 lds[];
  // Read the arguments in place (constant memory, uniform addresses): indexing the by-value
  // parameter would copy it to per-lane scratch.
  ConstProgArgs A = (ConstProgArgs)__builtin_amdgcn_kernarg_segment_ptr();
  const uint32_t rows = A->p.rows, cols = A->p.cols;
  const int n_regs = A->p.n_regs, n_sregs = A->p.n_sregs;
  const uint32_t tid = threadIdx.x;
  const uint32_t nvec = cols / VEC;
  const int n_col = A->p.n_col;
  f32x4* regs = lds;                                                    // [n_regs][CH][256], private to the lane
  f32x4* colfile = lds + (size_t)n_regs * CH * 256;                     // [n_col][nvec][VEC/4], shared by the workgroup
  float* sregs = reinterpret_cast<float*>(colfile + (size_t)n_col * nvec * (VEC / 4));   // [n_sregs][256]
  float* slots = sregs + (size_t)n_sregs * 256;                         // [kProgMaxReductions][4]

  const bool block_mode = A->p.lanes_per_row > 64;
  uint32_t L, lane, row;
  if (block_mode) {
    L = 256;
    lane = tid;
    row = blockIdx.x;
  } else {
    L = (uint32_t)A->p.lanes_per_row;
    lane = tid & (L - 1);
    row = blockIdx.x * (256u >> A->p.lanes_log2) + (tid >> A->p.lanes_log2);
  }
  const bool row_ok = row < rows;
  const bool row_full = nvec == L * (uint32_t)K;
  const uint32_t row_c = min(row, rows - 1);
  const size_t base = (size_t)row_c * cols;
  auto valid = [&](int k) { return lane + k * L < nvec; };
  auto vec_at = [&](int k) { return min(lane + k * L, nvec - 1); };
  auto put = [&](int reg, const float (&v)[KV]) {
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const f32x4 t = {v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]};
      regs[((uint32_t)reg * CH + j) * 256u + tid] = t;
    }
  };
  auto get = [&](int reg, float (&v)[KV]) {
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const f32x4 t = regs[((uint32_t)reg * CH + j) * 256u + tid];
      v[4 * j] = t.x; v[4 * j + 1] = t.y; v[4 * j + 2] = t.z; v[4 * j + 3] = t.w;
    }
  };

  // the program itself: one instruction per lane (kProgMaxInstr == 64 lanes of a wavefront)
  const int n_instr = A->p.n_instr;
  uint32_t iw0, iw1, iw2;
  {
    const uint32_t slot = min(tid & 63u, (uint32_t)max(n_instr - 1, 0));
    const uint32_t __attribute__((address_space(4)))* w =
        reinterpret_cast<const uint32_t __attribute__((address_space(4)))*>(&A->p.instr[slot]);
    iw0 = w[0]; iw1 = w[1]; iw2 = w[2];
  }

  float acc[KV];
#pragma unroll
  for (int j = 0; j < KV; ++j) acc[j] = 0.0f;
  const int acc_input = A->p.acc_input;

  // the row's index along the pattern's (collapsed) leading axes, for inputs stretched along some of them and for
  // inputs / outputs whose rows are renumbered by a folded transpose
  uint32_t c0 = 0, c1 = 0, c2 = 0;
  // ---- prologue: every global load is issued before anything waits ------------------------
  // full-shaped inputs are parked in registers of the per-lane file; column vectors are unpacked
  // once per workgroup into the shared column file; per-row scalar inputs go to the scalar file.
  {
    const int n_full = A->p.n_full;
    if (A->p.full_bcast | A->p.rscal_bcast | A->p.out_perm) {
      const FastDiv od1 = {A->p.od[1].d, A->p.od[1].m, A->p.od[1].s}, od2 = {A->p.od[2].d, A->p.od[2].m, A->p.od[2].s};
      const uint32_t r1 = fast_div(row_c, od2);
      c2 = row_c - r1 * od2.d;
      c0 = fast_div(r1, od1);
      c1 = r1 - c0 * od1.d;
    }
    RawVec<VEC, VEC / 4> raw[NI][K];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      if (i < n_full) {
        const int dt = A->p.full_dt[i];
        size_t base_i = base;
        if ((A->p.full_bcast >> i) & 1u)   // stretched along leading axes: its own row index
          base_i = (size_t)(c0 * A->p.ms[i][0] + c1 * A->p.ms[i][1] + c2 * A->p.ms[i][2]) * cols;
#pragma unroll
        for (int k = 0; k < K; ++k) raw[i][k] = load_elems<VEC>(A->full[i], base_i + (size_t)vec_at(k) * VEC, dt, true);
      }
    }
    const int n_rscal = A->p.n_rscal;
    float rs[kProgMaxOperands];
#pragma unroll
    for (int i = 0; i < kProgMaxOperands; ++i) {
      if (i < n_rscal) {
        size_t at = row_c;
        if ((A->p.rscal_bcast >> i) & 1u) at = c0 * A->p.rms[i][0] + c1 * A->p.rms[i][1] + c2 * A->p.rms[i][2];
        rs[i] = load_scalar_as(A->rscal[i], at, A->p.rscal_dt[i]);
      }
    }
    for (int i = 0; i < n_col; ++i) {
      const int dt = A->p.col_dt[i];
      for (uint32_t j = tid; j < nvec; j += 256u) {
        float part[VEC];
        unpack_elems<VEC>(load_elems<VEC>(A->col[i], (size_t)j * VEC, dt, false), dt, part);
#pragma unroll
        for (int h = 0; h < VEC / 4; ++h) {
          const f32x4 t = {part[4 * h], part[4 * h + 1], part[4 * h + 2], part[4 * h + 3]};
          colfile[((uint32_t)i * nvec + j) * (VEC / 4) + h] = t;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < kProgMaxOperands; ++i) {
      if (i < n_rscal) sregs[(uint32_t)A->p.rscal_sreg[i] * 256u + tid] = rs[i];
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      if (i < n_full) {
        float v[KV];
        const int dt = A->p.full_dt[i];
#pragma unroll
        for (int k = 0; k < K; ++k) {
          float part[VEC];
          unpack_elems<VEC>(raw[i][k], dt, part);
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[k * VEC + e] = part[e];
        }
        if (A->p.full_reg[i] != 255) put(A->p.full_reg[i], v);
        if (i == acc_input) {
#pragma unroll
          for (int j = 0; j < KV; ++j) acc[j] = v[j];
        }
      }
    }
    if (n_col > 0) __syncthreads();   // n_col is uniform: every thread of the workgroup arrives
  }

  // ---- instruction walk: an accumulator machine ----------------------------------------------
  // full-shaped:  acc <- acc (op) b | (op) acc | b      per-row:  sacc <- sacc (op) b | (op) sacc | b
  // b comes from a register, the column file, a per-row scalar (stretched along the row) or the
  // immediate; PF_KEEP also writes the result to a register.
  float sacc = 0.0f;
  int reduction_no = 0;
  for (int pc = 0; pc < n_instr; ++pc) {
    // lane i of every wavefront holds instruction i: fetching one is three cross-lane reads
    // into scalar registers, with no memory latency inside the walk
    const uint32_t w0 = (uint32_t)__builtin_amdgcn_readlane((int)iw0, pc);
    const uint32_t w1 = (uint32_t)__builtin_amdgcn_readlane((int)iw1, pc);
    const float imm = __builtin_bit_cast(float, __builtin_amdgcn_readlane((int)iw2, pc));
    const uint32_t op = w0 & 0xFF, b_kind = (w0 >> 8) & 0xFF, flags = (w0 >> 16) & 0xFF;
    const uint32_t b_idx = w1 & 0xFF, dst = (w1 >> 8) & 0xFF, aux = (w1 >> 16) & 0xFF;

    if (op == PO_STORE) {
      void* out = A->out[dst];
      size_t out_row = row;
      if ((A->p.out_perm >> dst) & 1u) out_row = (size_t)(c0 * A->p.oms[dst][0] + c1 * A->p.oms[dst][1] + c2 * A->p.oms[dst][2]);
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float part[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) part[e] = acc[k * VEC + e];
        if (row_ok && valid(k)) {
          const size_t at = out_row * cols + (size_t)(lane + k * L) * VEC;
          if (aux == DT_F32) StoreN<float, VEC>::run(static_cast<float*>(out) + at, part);
          else if (aux == DT_F16) StoreN<f16_t, VEC>::run(static_cast<f16_t*>(out) + at, part);
          else StoreN<bf16_t, VEC>::run(static_cast<bf16_t*>(out) + at, part);
        }
      }
    } else if (op == PO_STORE_SCAL) {
      if (row_ok && lane == 0) store_scalar_as(A->rout[dst], row, (int)aux, sacc);
    } else if (op == PO_RSUM || op == PO_RMAX || op == PO_RSUMSQ) {
      const bool is_max = op == PO_RMAX;
      const bool squared = op == PO_RSUMSQ;
      float r = is_max ? -INFINITY : 0.0f;
      if (row_full) {   // the row fills its lanes exactly: no padding slot to leave out
#pragma unroll
        for (int j = 0; j < KV; ++j) {
          const float x = squared ? acc[j] * acc[j] : acc[j];
          r = is_max ? fmaxf(r, x) : r + x;
        }
      } else {
#pragma unroll
        for (int k = 0; k < K; ++k) {
          const bool ok = valid(k);
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            const float v = acc[k * VEC + e];
            const float x = squared ? v * v : v;
            r = is_max ? fmaxf(r, ok ? x : -INFINITY) : r + (ok ? x : 0.0f);
          }
        }
      }
      if (block_mode) {
        float* slot = slots + 4 * reduction_no;
        r = is_max ? block_allreduce<OpMax>(r, slot, 4) : block_allreduce<OpSum>(r, slot, 4);
      } else {
        r = is_max ? group_allreduce<OpMax>(r, (int)L) : group_allreduce<OpSum>(r, (int)L);
      }
      ++reduction_no;
      sacc = r;
      if (flags & PF_KEEP) sregs[dst * 256u + tid] = r;
    } else if (flags & PF_SCALAR) {
      const float b = b_kind == PK_SCAL ? sregs[b_idx * 256u + tid] : (b_kind == PK_SACC ? sacc : imm);
      sacc = apply_op((int)op, sacc, b, (int)aux);
      if (flags & PF_KEEP) sregs[dst * 256u + tid] = sacc;
    } else {
      // one flat dispatch on (op, where b comes from): every case updates the accumulator in place and the
      // cases meet again in a single place, so the accumulator is not copied around between nested merges
      const uint32_t b_class = b_kind == PK_REG ? 1u : (b_kind == PK_COL ? 2u : (b_kind == PK_ACC ? 3u : 0u));
      const float sb = b_kind == PK_SCAL ? sregs[b_idx * 256u + tid] : (b_kind == PK_SACC ? sacc : imm);
      switch (op * 4u + b_class) {
#define FS_B_SCALAR(OP)                                                                \
  case (OP) * 4u + 0u:                                                                 \
    _Pragma("unroll") for (int j = 0; j < KV; ++j) acc[j] = apply_op(OP, acc[j], sb, (int)aux); \
    break;
#define FS_B_REG(OP)                                                                   \
  case (OP) * 4u + 1u: {                                                               \
    float b[KV];                                                                       \
    get((int)b_idx, b);                                                                \
    _Pragma("unroll") for (int j = 0; j < KV; ++j) acc[j] = apply_op(OP, acc[j], b[j], 0); \
    break;                                                                             \
  }
#define FS_B_COL(OP)                                                                   \
  case (OP) * 4u + 2u: {                                                               \
    _Pragma("unroll") for (int k = 0; k < K; ++k) {                                    \
      const f32x4* src = colfile + (b_idx * nvec + vec_at(k)) * (VEC / 4);             \
      _Pragma("unroll") for (int h = 0; h < VEC / 4; ++h) {                            \
        const f32x4 t = src[h];                                                        \
        const int j = k * VEC + 4 * h;                                                 \
        acc[j] = apply_op(OP, acc[j], t.x, 0);                                         \
        acc[j + 1] = apply_op(OP, acc[j + 1], t.y, 0);                                 \
        acc[j + 2] = apply_op(OP, acc[j + 2], t.z, 0);                                 \
        acc[j + 3] = apply_op(OP, acc[j + 3], t.w, 0);                                 \
      }                                                                                \
    }                                                                                  \
    break;                                                                             \
  }
#define FS_B_ACC(OP)                                                                   \
  case (OP) * 4u + 3u:                                                                 \
    _Pragma("unroll") for (int j = 0; j < KV; ++j) acc[j] = apply_op(OP, acc[j], acc[j], 0); \
    break;
#define FS_BINARY(OP) FS_B_SCALAR(OP) FS_B_REG(OP) FS_B_COL(OP) FS_B_ACC(OP)
        FS_BINARY(PO_ADD) FS_BINARY(PO_SUB) FS_BINARY(PO_RSUB) FS_BINARY(PO_MUL) FS_BINARY(PO_DIV) FS_BINARY(PO_RDIV)
        FS_BINARY(PO_MAX) FS_BINARY(PO_LOAD)
        FS_B_SCALAR(PO_SQUARE) FS_B_SCALAR(PO_EXP) FS_B_SCALAR(PO_RSQRT) FS_B_SCALAR(PO_TANH) FS_B_SCALAR(PO_GELU)
        FS_B_SCALAR(PO_GELU_GRAD) FS_B_SCALAR(PO_CVT)
        FS_B_SCALAR(PO_LOG) FS_B_SCALAR(PO_SIGMOID) FS_B_SCALAR(PO_RELU) FS_B_SCALAR(PO_ABS) FS_B_SCALAR(PO_SQRT)
#undef FS_BINARY
#undef FS_B_ACC
#undef FS_B_COL
#undef FS_B_REG
#undef FS_B_SCALAR
        default:
          break;
      }
    }
    if (!(flags & PF_SCALAR) && op <= PO_LOAD && (flags & PF_KEEP)) put((int)dst, acc);
  }
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <int VEC, int NI>
const void* prog_sym_k(int K) {
  switch (K) {
    case 1: return (const void*)k_row_program<VEC, 1, NI>;
    case 2: return (const void*)k_row_program<VEC, 2, NI>;
    case 4: return (const void*)k_row_program<VEC, 4, NI>;
    default: return nullptr;
  }
}
template <int VEC>
const void* prog_sym(int K, int n_full) {
  if (n_full <= 1) return prog_sym_k<VEC, 1>(K);
  if (n_full <= 2) return prog_sym_k<VEC, 2>(K);
  return prog_sym_k<VEC, 4>(K);
}
}  // namespace

const void* rowprog_kernel_symbol(int32_t, const KernelArgs& a) {
  const RowProgP& p = a.u.prog;
  if (p.n_full < 0 || p.n_full > kProgMaxInterpretedFull) return nullptr;
  if (p.vec == 4) return prog_sym<4>(p.vecs_per_lane, p.n_full);
  if (p.vec == 8) return prog_sym<8>(p.vecs_per_lane, p.n_full);
  return nullptr;
}

}  // namespace fs
