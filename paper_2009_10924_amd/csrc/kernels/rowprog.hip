// Interpreted row program: the generic code path for fusion patterns no hand-written
// kernel family covers (paper Section 4: any pattern of memory-intensive ops whose reuse
// stays inside a warp or a block is one kernel).  A pattern of element-wise ops,
// broadcasts and last-axis reductions over one [rows, cols] space is compiled on the host
// into a short instruction list; this kernel executes it with
//   * a row per lane group of one wavefront (warp composition) or per workgroup (block
//     composition), exactly like the hand-written row kernels,
//   * every global load issued before the first instruction runs, each input read once,
//   * column vectors in an LDS file shared by the workgroup; full-shaped values in an
//     accumulator (VGPRs) or a per-lane register file in LDS (a lane only ever touches its own
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

__device__ __forceinline__ float apply_op(int op, float a, float b, int aux) {
  switch (op) {
    case PO_ADD: return a + b;
    case PO_SUB: return a - b;
    case PO_MUL: return a * b;
    case PO_DIV: return a * fast_rcp(b);
    case PO_MAX: return fmaxf(a, b);
    case PO_SQUARE: return a * a;
    case PO_EXP: return fast_exp(a);
    case PO_RSQRT: return fast_rsqrt(a);
    case PO_TANH: return tanhf(a);
    case PO_GELU: return gelu_fwd(a);
    case PO_GELU_GRAD: return gelu_grad(a);
    case PO_CVT: return round_through(a, aux);
    default: return a;   // PO_MOV
  }
}

// NI: capacity for full-shaped inputs (sizes the prologue's load batch).
template <typename T, int K, int NI>
__global__ void __launch_bounds__(256) k_row_program(const ProgArgs args_in_kernarg) {
  constexpr int VEC = Elem<T>::VEC;
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
  const uint32_t row_c = min(row, rows - 1);
  const size_t base = (size_t)row_c * cols;
  auto valid = [&](int k) { return lane + k * L < nvec; };
  auto vec_at = [&](int k) { return min(lane + k * L, nvec - 1); };
  auto put = [&](int reg, const float (&v)[KV]) {
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const f32x4 t = {v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]};
      regs[((size_t)reg * CH + j) * 256 + tid] = t;
    }
  };
  auto get = [&](int reg, float (&v)[KV]) {
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const f32x4 t = regs[((size_t)reg * CH + j) * 256 + tid];
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

  // ---- prologue: every global load is issued before anything waits ------------------------
  // full-shaped inputs are parked in registers of the per-lane file; column vectors are unpacked
  // once per workgroup into the shared column file; per-row scalar inputs go to the scalar file.
  {
    const int n_full = A->p.n_full;
    u32x4 raw[NI][K];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      if (i < n_full) {
        const T* src = static_cast<const T*>(A->full[i]) + base;
#pragma unroll
        for (int k = 0; k < K; ++k) raw[i][k] = load_raw_nt(src + (size_t)vec_at(k) * VEC);
      }
    }
    const int n_rscal = A->p.n_rscal;
    float rs[kProgMaxOperands];
#pragma unroll
    for (int i = 0; i < kProgMaxOperands; ++i) {
      if (i < n_rscal) rs[i] = load_scalar_as(A->rscal[i], row_c, A->p.rscal_dt[i]);
    }
    for (int i = 0; i < n_col; ++i) {
      const T* src = static_cast<const T*>(A->col[i]);
      for (uint32_t j = tid; j < nvec; j += 256u) {
        float part[VEC];
        unpack(load_raw(src + (size_t)j * VEC), part, (const T*)nullptr);
#pragma unroll
        for (int h = 0; h < VEC / 4; ++h) {
          const f32x4 t = {part[4 * h], part[4 * h + 1], part[4 * h + 2], part[4 * h + 3]};
          colfile[((size_t)i * nvec + j) * (VEC / 4) + h] = t;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < kProgMaxOperands; ++i) {
      if (i < n_rscal) sregs[(size_t)A->p.rscal_sreg[i] * 256 + tid] = rs[i];
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      if (i < n_full) {
        float v[KV];
#pragma unroll
        for (int k = 0; k < K; ++k) {
          float part[VEC];
          unpack(raw[i][k], part, (const T*)nullptr);
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[k * VEC + e] = part[e];
        }
        put(A->p.full_reg[i], v);
      }
    }
    if (n_col > 0) __syncthreads();   // n_col is uniform: every thread of the workgroup arrives
  }

  // ---- instruction walk -------------------------------------------------------------------
  float acc[KV];
#pragma unroll
  for (int j = 0; j < KV; ++j) acc[j] = 0.0f;
  float sacc = 0.0f;
  int reduction_no = 0;
  for (int pc = 0; pc < n_instr; ++pc) {
    // lane i of every wavefront holds instruction i (loaded once, below): fetching one is three
    // cross-lane reads into scalar registers, with no memory latency inside the walk
    const uint32_t w0 = (uint32_t)__builtin_amdgcn_readlane((int)iw0, pc);
    const uint32_t w1 = (uint32_t)__builtin_amdgcn_readlane((int)iw1, pc);
    const uint32_t w2 = (uint32_t)__builtin_amdgcn_readlane((int)iw2, pc);
    ProgInstr ins;
    ins.op = w0 & 0xFF; ins.a_kind = (w0 >> 8) & 0xFF; ins.b_kind = (w0 >> 16) & 0xFF; ins.flags = w0 >> 24;
    ins.a = w1 & 0xFF; ins.b = (w1 >> 8) & 0xFF; ins.dst = (w1 >> 16) & 0xFF; ins.aux = w1 >> 24;
    ins.imm = __builtin_bit_cast(float, w2);
    auto scalar_operand = [&](int kind, int idx) {
      if (kind == PK_SACC) return sacc;
      if (kind == PK_SCAL) return sregs[(size_t)idx * 256 + tid];
      return ins.imm;
    };
    auto vector_operand = [&](int kind, int idx, float (&v)[KV]) {
      if (kind == PK_ACC) {
#pragma unroll
        for (int j = 0; j < KV; ++j) v[j] = acc[j];
      } else if (kind == PK_REG) {
        get(idx, v);
      } else if (kind == PK_COL) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
          const f32x4* src = colfile + ((size_t)idx * nvec + vec_at(k)) * (VEC / 4);
#pragma unroll
          for (int h = 0; h < VEC / 4; ++h) {
            const f32x4 t = src[h];
            v[k * VEC + 4 * h] = t.x; v[k * VEC + 4 * h + 1] = t.y; v[k * VEC + 4 * h + 2] = t.z; v[k * VEC + 4 * h + 3] = t.w;
          }
        }
      } else {
        const float s = scalar_operand(kind, idx);
#pragma unroll
        for (int j = 0; j < KV; ++j) v[j] = s;
      }
    };

    if (ins.op == PO_STORE) {
      float v[KV];
      vector_operand(ins.a_kind, ins.a, v);
      void* out = A->out[ins.dst];
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float part[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) part[e] = v[k * VEC + e];
        if (row_ok && valid(k)) {
          const size_t at = (size_t)row * cols + (size_t)(lane + k * L) * VEC;
          if (ins.aux == DT_F32) StoreN<float, VEC>::run(static_cast<float*>(out) + at, part);
          else if (ins.aux == DT_F16) StoreN<f16_t, VEC>::run(static_cast<f16_t*>(out) + at, part);
          else StoreN<bf16_t, VEC>::run(static_cast<bf16_t*>(out) + at, part);
        }
      }
    } else if (ins.op == PO_STORE_SCAL) {
      const float s = scalar_operand(ins.a_kind, ins.a);
      if (row_ok && lane == 0) store_scalar_as(A->rout[ins.dst], row, ins.aux, s);
    } else if (ins.op == PO_RSUM || ins.op == PO_RMAX) {
      float v[KV];
      vector_operand(ins.a_kind, ins.a, v);
      const bool is_max = ins.op == PO_RMAX;
      float r = is_max ? -INFINITY : 0.0f;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const bool ok = valid(k);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float x = v[k * VEC + e];
          r = is_max ? fmaxf(r, ok ? x : -INFINITY) : r + (ok ? x : 0.0f);
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
      if (ins.flags & PF_KEEP) sregs[(size_t)ins.dst * 256 + tid] = r;
    } else if (ins.flags & PF_SCALAR) {
      const float a = scalar_operand(ins.a_kind, ins.a);
      const float b = scalar_operand(ins.b_kind, ins.b);
      sacc = apply_op(ins.op, a, b, ins.aux);
      if (ins.flags & PF_KEEP) sregs[(size_t)ins.dst * 256 + tid] = sacc;
    } else {
      float a[KV], b[KV];
      vector_operand(ins.a_kind, ins.a, a);
      if (ins.op <= PO_MAX) {
        vector_operand(ins.b_kind, ins.b, b);
      } else {
#pragma unroll
        for (int j = 0; j < KV; ++j) b[j] = 0.0f;
      }
      // the op is uniform: one scalar branch per instruction, then straight-line lane work
      switch (ins.op) {
#define FS_PROG_CASE(OP)                                                            \
  case OP:                                                                          \
    _Pragma("unroll") for (int j = 0; j < KV; ++j) acc[j] = apply_op(OP, a[j], b[j], ins.aux); \
    break;
        FS_PROG_CASE(PO_ADD) FS_PROG_CASE(PO_SUB) FS_PROG_CASE(PO_MUL) FS_PROG_CASE(PO_DIV) FS_PROG_CASE(PO_MAX)
        FS_PROG_CASE(PO_SQUARE) FS_PROG_CASE(PO_EXP) FS_PROG_CASE(PO_RSQRT) FS_PROG_CASE(PO_TANH)
        FS_PROG_CASE(PO_GELU) FS_PROG_CASE(PO_GELU_GRAD) FS_PROG_CASE(PO_CVT)
#undef FS_PROG_CASE
        default:
#pragma unroll
          for (int j = 0; j < KV; ++j) acc[j] = a[j];
          break;
      }
      if (ins.flags & PF_KEEP) put(ins.dst, acc);
    }
  }
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <typename T, int NI>
const void* prog_sym_k(int K) {
  switch (K) {
    case 1: return (const void*)k_row_program<T, 1, NI>;
    case 2: return (const void*)k_row_program<T, 2, NI>;
    case 4: return (const void*)k_row_program<T, 4, NI>;
    default: return nullptr;
  }
}
template <typename T>
const void* prog_sym(int K, int n_full) {
  if (n_full <= 1) return prog_sym_k<T, 1>(K);
  if (n_full <= 2) return prog_sym_k<T, 2>(K);
  return prog_sym_k<T, 4>(K);
}
}  // namespace

const void* rowprog_kernel_symbol(int32_t, const KernelArgs& a) {
  const RowProgP& p = a.u.prog;
  if (p.n_full < 0 || p.n_full > kProgMaxOperands) return nullptr;
  switch (p.dt) {
    case DT_F32: return prog_sym<float>(p.vecs_per_lane, p.n_full);
    case DT_F16: return prog_sym<f16_t>(p.vecs_per_lane, p.n_full);
    case DT_BF16: return prog_sym<bf16_t>(p.vecs_per_lane, p.n_full);
    default: return nullptr;
  }
}

}  // namespace fs
