// Host-visible description of every kernel the library can launch: ids, parameter
// blocks (plain data, passed by value), launch shapes.  No HIP types here so the
// host-only translation units can include it.
#pragma once
#include <cstdint>
#include <memory>
#include <string>

namespace fs {

constexpr int kMaxPtrs = 44;
// Pointer slots of a row program (interpreted or generated): kProgMaxOperands each of full-shaped inputs, column
// vectors, per-row scalar inputs, full-shaped outputs, per-row outputs, then the workspace of a generated kernel.
constexpr int kSlotFull = 0, kSlotCol = 8, kSlotRscal = 16, kSlotOut = 24, kSlotRout = 32, kSlotWs = 40;
constexpr int kGenArgPtrs = 41;   // pointers of a generated kernel: the operand slots + the workspace

// storage dtypes, numbered like the public fs_dtype
enum DType : int32_t { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2, DT_I32 = 3 };

enum KernelId : int32_t {
  // per-op baseline
  K_UNARY = 0,         // p0 in, p1 out
  K_BINARY,            // p0 a, p1 b, p2 out
  K_REDUCE_ROW,        // p0 in [rows, cols], p1 out [rows]
  K_REDUCE_MID,        // p0 in [outer, red, inner], p1 out [outer, nchunk, inner]
  K_TRANSPOSE_ROWS,    // p0 in, p1 out : permutation keeps the innermost axis
  K_TRANSPOSE_TILE,    // p0 in, p1 out : innermost axis moves, staged through an LDS tile
  K_COPY,              // p0 src, p1 dst
  // stitched
  K_SOFTMAX_WAVE,      // p0 x, p1 mask (or null), p2 out
  K_SOFTMAX_BLOCK,     // same operands, one workgroup per row, reduced values through LDS
  K_LAYERNORM_WAVE,    // p0 x, p1 res, p2 bias, p3 gamma, p4 beta, p5 out, p6 row mean out (or null), p7 row rstd out (or null)
  K_LAYERNORM_BLOCK,
  K_BIAS_GELU,         // p0 x, p1 bias, p2 y
  K_BIAS_GELU_DBIAS,   // p0 x, p1 bias, p2 grad, p3 y, p4 partials [n_row_tiles, cols] f32 (folded by K_COLFOLD)
  K_COLFOLD,           // p0 partials [n_row_tiles, fold_cols] f32, p1 out0 (columns < fold_split), p2 out1 (the rest), both of dtype dt
  K_TCHAIN_WAVE,       // p0 x, p1 scale, p2 out
  K_TCHAIN_LDS,
  K_ROW_WAVE,          // p0,p1 row inputs, p2,p3 column vectors, p4 out0, p5 out1 : generic row-stitched skeleton
  K_ROW_BLOCK,         // same operands as K_ROW_WAVE, one workgroup per row, reduced values through LDS
  K_ROW_PROGRAM,       // interpreted row program: p0-7 full inputs, p8-15 column vectors, p16-23 per-row scalar
                       // inputs, p24-31 full outputs, p32-39 per-row scalar outputs (kSlot*)
  K_LAYERNORM_BWD,     // p0 h, p1 dy, p2 gamma, p3 mu, p4 rstd, p5 dx, p6 partials [n_row_blocks, 2, cols]
  K_ROW_GENERATED,     // a kernel generated and compiled for one row pattern at plan time; pointer slots as K_ROW_PROGRAM,
                       // p40 the workspace for column partial sums (or null).
                       // Not in the compiled-in table: launched through its own handle (gen_launch)
  K_COUNT
};

// Division of a 31-bit index by a run-time constant as multiply-high + shift:
// q = n (d == 1), else q = mulhi(n, m) >> s with m = floor(2^(32+s) / d) + 1, s = ceil(log2 d) - 1.
struct FastDiv {
  uint32_t d, m, s;
};

struct LaunchShape {
  uint32_t grid[3] = {1, 1, 1};
  uint32_t block[3] = {1, 1, 1};
  uint32_t lds_bytes = 0;   // dynamic LDS
};

// ---- per-op baseline ----------------------------------------------------------
enum UnaryOp : int32_t { U_COPY = 0, U_SCALE, U_ADD_SCALAR, U_SQUARE, U_EXP, U_RSQRT, U_TANH, U_GELU, U_GELU_GRAD, U_LOG, U_SIGMOID, U_RELU, U_ABS, U_SQRT };
struct UnaryP {
  int32_t op, in_dt, out_dt, vec;   // vec: elements per lane per step (8, 4 or 1)
  uint32_t n;
  float value;
};
enum BinaryOp : int32_t { B_ADD = 0, B_SUB, B_MUL, B_DIV, B_MAX, B_FIRST };
struct BinaryP {
  int32_t op, a_dt, b_dt, out_dt, vec, rank;
  uint32_t n;            // output elements
  uint32_t dims[4];      // collapsed output extents, dims[rank-1] innermost
  uint32_t sa[4], sb[4]; // operand strides in elements (0 = broadcast)
};
enum ReduceOp : int32_t { R_SUM = 0, R_MAX, R_MEAN };
struct ReduceP {
  int32_t op, in_dt, out_dt, vec;
  uint32_t outer, red, inner;   // input viewed as [outer, red, inner]
  uint32_t chunk, nchunk;       // K_REDUCE_MID: rows of `red` per workgroup, chunks per column
  uint32_t lanes_per_row;       // K_REDUCE_ROW
  float post_scale;             // 1/red for mean on the final pass, else 1
};
struct TransposeP {
  int32_t elem_bytes, vec;      // vec: elements per 128-bit (or narrower) access along the inner axis
  uint32_t out_dims[4];         // output extents padded to rank 4 (leading 1s)
  uint32_t in_stride[4];        // input stride (elements) of the axis that feeds each output axis
  uint32_t n;
  // K_TRANSPOSE_TILE: the two axes of the tile
  uint32_t tile_in_axis_out_pos;  // output position of the input's innermost axis
  uint32_t out_stride[4];
  uint32_t tile_uq;               // vectorised tile: 16-byte units along the input's innermost axis (16 or 8); the tile is
                                  // tile_uq * vec elements along it by (256 / tile_uq) * vec along the output's innermost axis
  uint32_t order;                 // which index neighbouring workgroups differ in: 0 the tile along the output's innermost
                                  // axis, 1 the inner one of the two axes outside the tile
};

// ---- stitched -----------------------------------------------------------------
struct SoftmaxP {
  int32_t in_dt, out_dt, mask_dt;
  int32_t has_mask, mask_inner;     // mask_inner: 1 if the mask varies along the row, 0 if one value per row
  uint32_t rows, cols;
  FastDiv od[3];                    // outer extents of the row index (od[2] fastest), product = rows
  uint32_t ms[3];                   // mask element stride for each outer coordinate
  float scale;
  int32_t lanes_per_row, vecs_per_lane;
  int32_t lanes_log2;               // log2(lanes_per_row) for the wave variant
  int32_t fast;                     // 1: the row fills the lanes and the rows fill the workgroups exactly
};
struct LayerNormP {
  int32_t in_dt, out_dt, par_dt;    // x/res dtype, output dtype, bias/gamma/beta dtype
  int32_t has_res, has_bias, has_affine;
  int32_t stats;                    // 1: the per-row mean / rstd pointers are live
  uint32_t rows, cols;
  float eps, inv_cols;              // inv_cols = 1 / cols, rounded on the host
  int32_t lanes_per_row, vecs_per_lane, rows_per_block;
  int32_t lanes_log2;
  int32_t fast;                     // 1: all operands present, row and row count fill lanes / workgroups exactly
};
struct GeluP {
  int32_t dt, bias_dt;              // x / grad / y share dt; K_COLFOLD: dt = dtype the sums are handed out in
  uint32_t rows, cols;              // K_COLFOLD: cols = floats between two partial rows
  uint32_t n_row_tiles;             // row blocks = rows of the partials workspace
  int32_t waves, unroll;            // workgroup = waves x 64 lanes; a row tile = waves * unroll rows
  int32_t fast;                     // 1: rows fill every workgroup's row tiles and cols fill the column tiles exactly
  uint32_t fold_cols, fold_split;   // K_COLFOLD: columns of the partials, first column that goes to the second output
  uint32_t fold_quads;              // K_COLFOLD: column quads per workgroup (16 with 16 row groups, or 4 with 64)
};
struct TChainP {
  int32_t dt, scale_dt;
  uint32_t B, S, H, D;              // input [B,S,H,D] -> output [B,H,S,D]
  float eps;
  int32_t lanes_per_row, vecs_per_lane, s_tile;
  int32_t passes;                   // rows each lane group handles = ceil(s_tile * H / groups), 1..4
  int32_t lanes_log2;
  FastDiv div_h, div_s_tiles;       // division by H and by the number of s tiles per batch entry
};

struct LnBwdP {
  int32_t dt;                       // h / dy / gamma / dx share dt; mu, rstd, dgamma, dbeta are float32
  uint32_t rows, cols;
  float inv_cols;
  int32_t lanes_per_row, lanes_log2, vecs_per_lane;
  int32_t waves, rows_per_group;    // workgroup = waves x 64 lanes; rows each lane group loads up front
  int32_t fast;                     // 1: the row fills the lanes exactly, the tiles fill the workgroups' rounds exactly
};
enum RowPattern : int32_t { ROW_SOFTMAX_BWD = 0, ROW_RMSNORM = 1 };
struct RowP {
  int32_t pattern, dt;              // all row inputs and outputs share dt
  uint32_t rows, cols;
  float f[4];                       // pattern scalars
  int32_t lanes_per_row, lanes_log2, vecs_per_lane, fast;
};

// ---- packed launch: many independent row patterns in one kernel -----------------------
enum PackSpec : int32_t {
  PACK_SOFTMAX = 0,      // in0 x;                                  f[0] = scale
  PACK_SOFTMAX_BWD = 1,  // in0 y, in1 dy
  PACK_RMSNORM = 2,      // in0 x, vec0 gamma;                      f[0] = eps, f[1] = 1/cols
  PACK_LN_FULL = 3,      // in0 x, in1 res, vec0 bias, vec1 gamma, vec2 beta; f as above
  PACK_LN_PLAIN = 4,     // in0 x, vec0 gamma, vec1 beta;           f as above
  PACK_BIAS_GELU = 5,    // in0 x, vec0 bias
  PACK_SPEC_COUNT = 6
};
// dtype pairs (storage of inputs -> storage of the output) the packed kernel is compiled for
enum PackTypes : int32_t { PT_F32 = 0, PT_F16 = 1, PT_BF16 = 2, PT_F32_BF16 = 3, PT_COUNT = 4 };
constexpr int kPackMaxMembers = 32;   // one launch; the table travels in the kernel arguments
struct PackEntry {
  const void* in[2];
  const void* vec[3];
  void* out;
  RowP p;                // lanes_per_row > 64: one workgroup per row; p.pattern holds the PackSpec
  int32_t variant;       // (spec * PT_COUNT + types) * 3 + log2(vecs_per_lane)
  int32_t reserved;
};
struct PackTable {
  // first workgroup of the launch that serves member j, ascending; unused slots hold 0xFFFFFFFF.
  // Kept together at the front so a workgroup finds its member from two wide scalar loads.
  uint32_t first_block[kPackMaxMembers];
  int32_t n;
  uint32_t total_blocks;
  PackEntry e[kPackMaxMembers];
};
// ---- interpreted row program -------------------------------------------------------------
// Any connected pattern of element-wise ops, broadcasts and last-axis reductions over one
// [rows, cols] space runs as ONE kernel: a lane group (or the workgroup) owns a row, values
// live in a per-lane register file in LDS plus an accumulator in VGPRs, and the kernel
// walks a short instruction list carried in its arguments.
enum ProgOp : uint8_t {
  PO_ADD = 0, PO_SUB, PO_RSUB, PO_MUL, PO_DIV, PO_RDIV, PO_MAX,   // acc (op) b;  RSUB = b - acc, RDIV = b / acc
  PO_SQUARE, PO_EXP, PO_RSQRT, PO_TANH, PO_GELU, PO_GELU_GRAD,    // (op) acc
  PO_LOG, PO_SIGMOID, PO_RELU, PO_ABS, PO_SQRT,
  PO_CVT,                                                 // acc rounded through storage dtype `aux`
  PO_LOAD,                                                // acc <- b
  PO_RSUM, PO_RMAX, PO_RSUMSQ,                            // row reduction of acc (RSUMSQ: of acc squared) -> sacc
  PO_STORE,                                               // acc -> full output `dst`, stored as dtype `aux`
  PO_STORE_SCAL,                                          // sacc -> per-row output `dst`, dtype `aux`
  PO_COLSUM                                               // acc is added to column sum `dst` (the sum over all rows of the
                                                          // pattern; generated kernels only: partial sums per workgroup go
                                                          // to the workspace and a second launch folds them)
};
// where operand b comes from
enum ProgKind : uint8_t {
  PK_ACC = 0,   // the accumulator itself (x (op) x)
  PK_SACC,      // the scalar accumulator
  PK_REG,       // full-shaped register (LDS, private to the lane)
  PK_SCAL,      // per-row scalar register
  PK_IMM,       // the instruction's immediate
  PK_COL        // column vector, from the workgroup's shared column file
};
enum ProgFlags : uint8_t {
  PF_SCALAR = 1,   // per-row-shaped instruction: works on sacc
  PF_KEEP = 2      // also write the result to register `dst` (full or scalar file by shape)
};
struct ProgInstr {
  uint8_t op, b_kind, flags, pad0;
  uint8_t b, dst, aux, pad1;
  float imm;
};
constexpr int kProgMaxInstr = 64;
constexpr int kProgMaxOperands = 8;     // per class: full inputs, column vectors, per-row inputs, outputs
constexpr int kProgMaxInterpretedFull = 4;   // full-shaped inputs the interpreter's load batch is built for
constexpr int kProgMaxColSums = 4;      // one fold launch hands out two: at most two fold launches
constexpr int kProgMaxReductions = 8;   // LDS slot sets of the workgroup-per-row form
constexpr int kProgMaxLdsBytes = 128 * 1024;   // register files of one workgroup (a CU has 160 KB)
struct RowProgP {
  int32_t vec;                         // elements a lane holds per 128-bit step of the narrowest vector input: 4 or 8
                                       // (a float32 input of a vec-8 program takes two 128-bit loads per step)
  uint32_t rows, cols;
  int32_t lanes_per_row, lanes_log2, vecs_per_lane;   // lanes_per_row > 64: one workgroup per row
  int32_t n_full, n_col, n_rscal, n_instr;
  int32_t n_regs, n_sregs;             // register files: full-shaped and per-row
  int32_t acc_input;                   // full-shaped input the accumulator starts out holding, -1 = none
  uint8_t full_reg[kProgMaxOperands];  // register each full-shaped input is parked in, 255 = not parked
  uint8_t full_dt[kProgMaxOperands], col_dt[kProgMaxOperands];   // storage dtypes of the vector inputs
  // full-shaped inputs that are stretched along some leading axes (an attention mask [B,1,1,T] under scores
  // [B,H,S,T]): bit i of full_bcast set -> the row of input i is c0*ms[i][0] + c1*ms[i][1] + c2*ms[i][2] with
  // (c0, c1, c2) the row's index along the pattern's leading axes, od[] their extents (collapsed to three)
  uint32_t full_bcast;
  uint32_t ms[kProgMaxOperands][3];
  uint32_t rscal_bcast;                 // the same for per-row scalar inputs (a per-head value [H,1,1] under [B,H,S,T])
  uint32_t rms[kProgMaxOperands][3];
  FastDiv od[3];
  // full-shaped outputs stored through a transpose of the leading axes: bit i of out_perm set -> the pattern's
  // row (c0, c1, c2) is row c0*oms[i][0] + c1*oms[i][1] + c2*oms[i][2] of output i
  uint32_t out_perm;
  uint32_t oms[kProgMaxOperands][3];
  uint8_t rscal_sreg[kProgMaxOperands], rscal_dt[kProgMaxOperands];
  int32_t n_colsum;                    // column sums over all rows (generated kernels only), at most kProgMaxColSums
  int32_t rows_per_group;              // rows each lane group works through, one after the other (> 1 only with column sums:
                                       // fewer, longer partial sums)
  int32_t col_tiles;                   // > 1: a workgroup handles one of col_tiles column tiles of cols / col_tiles elements
                                       // (generated kernels for patterns with column sums and no row reduction)
  int32_t col_chunks;                  // > 1: a row too long for the lanes' registers is worked through in col_chunks pieces of
                                       // lanes_per_row * vecs_per_lane steps, once per row reduction and once more for the stores
  int32_t col_kept;                    // of those chunks, the first col_kept stay in registers in storage form after the first
                                       // pass (the later passes do not read them again)
  ProgInstr instr[kProgMaxInstr];
};
struct ProgArgs {
  const void* full[kProgMaxOperands];
  const void* col[kProgMaxOperands];
  const void* rscal[kProgMaxOperands];
  void* out[kProgMaxOperands];
  void* rout[kProgMaxOperands];
  RowProgP p;
};

struct KernelArgs {
  void* p[kMaxPtrs] = {};
  union {
    UnaryP unary;
    BinaryP binary;
    ReduceP reduce;
    TransposeP transpose;
    SoftmaxP softmax;
    LayerNormP layernorm;
    GeluP gelu;
    TChainP tchain;
    RowP row;
    LnBwdP lnbwd;
    RowProgP prog;
  } u;
  KernelArgs() { u.binary = BinaryP{}; }
};

// Up to kFoldManyMax K_COLFOLD jobs as one launch (each entry = that kernel's pointers and GeluP fields).
constexpr int kFoldManyMax = 8;
struct FoldManyP {
  const float* partials[kFoldManyMax];
  float* out0[kFoldManyMax];
  float* out1[kFoldManyMax];
  uint32_t first_block[kFoldManyMax];   // first workgroup of each job; [0] = 0, unused entries = 0xffffffff
  uint32_t n[kFoldManyMax], width[kFoldManyMax], stride[kFoldManyMax], split[kFoldManyMax], quads[kFoldManyMax];
  int32_t out_dt[kFoldManyMax];         // dtype the sums are handed out in
};
int launch_fold_many(const FoldManyP& table, uint32_t n_blocks, void* stream);

struct KernelResources {
  int32_t vgprs = 0;       // architected vector registers per lane
  int32_t static_lds = 0;  // bytes
  bool from_device = false;
};

// Implemented in kernels/*.hip.  Returns hipError_t as int (0 = success).
int launch_kernel(int32_t kernel, const KernelArgs& args, const LaunchShape& shape, void* stream);
// Register / LDS figures of the variant `launch_kernel` would pick for these args.
KernelResources kernel_resources(int32_t kernel, const KernelArgs& args);
// Packed launch (kernels/pack.hip): one kernel over table.total_blocks workgroups.
int launch_pack(const PackTable& table, void* stream);
KernelResources pack_kernel_resources();
const char* kernel_name(int32_t kernel);
const char* hip_error_text(int err);

// ---- kernels compiled at plan time (kernels/gen_runtime.hip) -------------------------------
struct GenKernel;   // a compiled code object and, per device, the loaded function
struct GenResources {
  int32_t vgprs = 0, static_lds = 0;
  int32_t scratch_bytes = 0, spilled_vgprs = 0;   // per-lane scratch memory: registers did not suffice
  int64_t code_bytes = 0;
};
// true if the run-time compiler can be loaded in this process
bool gen_available();
// Compiles `source` (HIP, one extern "C" kernel `entry`) for gfx950; needs no GPU.  Identical sources share one
// compiled kernel for the life of the process.  Returns 0 or a hipError_t; *log receives the compiler's messages.
int gen_compile(const std::string& source, const char* entry, std::shared_ptr<GenKernel>* out, std::string* log);
GenResources gen_resources(const GenKernel* k);
// Loads the kernel's module on the current device if there is one (otherwise the first launch does).
int gen_preload(GenKernel* k);
// Launches with `args` (args_bytes of by-value kernel arguments).  Returns hipError_t as int.
int gen_launch(GenKernel* k, const void* args, size_t args_bytes, const LaunchShape& shape, void* stream);

}  // namespace fs
