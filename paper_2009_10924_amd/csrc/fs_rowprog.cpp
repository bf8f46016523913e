// Host compiler for the interpreted row program: turns any pattern of element-wise ops,
// broadcasts and last-axis reductions over one [rows, cols] space into the instruction
// list the K_ROW_PROGRAM kernel walks (paper Section 4.2: the schedule of a pattern
// follows from its sub-roots -- here the row reductions -- and every other op is
// computed where its consumer needs it; Section 4.4: values shared between ops get
// on-chip storage by lifetime).
//
// Value classes, relative to the largest tensor of the pattern ([.., C], R rows):
//   FULL  same extents                      -> per-lane vector, in the accumulator or an LDS register
//   RSCAL same leading extents, last = 1    -> per-row scalar, scalar accumulator or scalar register
//   COL   [C] / [1,..,1,C]                  -> the same for every row: an input sits in the workgroup's shared
//                                              column file, an intermediate is handled like a FULL value
// The kernel is an accumulator machine: every instruction works on the accumulator of its shape
// (acc <- acc (op) b).  A first walk over the ops follows what the accumulators hold and marks
// the values that some reader finds overwritten; only those are also written to a register
// (PF_KEEP).  A second walk allocates registers by lifetime and emits.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "fs_internal.hpp"
#include "fs_stitch_util.hpp"

namespace fs {
namespace {

enum ValKind : int { V_NONE = 0, V_FULL, V_RSCAL, V_COL };

struct Val {
  int kind = V_NONE;
  int root = -1;        // tensor whose storage this value shares (itself unless an alias)
  int reg = -1;         // register index in the file of its shape, -1 = none
  int input_index = -1; // column input: its position in the shared column file
  int last_read = -1;   // index of the last op that reads the root
  bool keep = false;    // some reader finds the accumulator overwritten: the value needs a register
};

struct Compiler {
  const fs_graph& g;
  std::vector<Val> val;
  int rank = 0;
  int64_t dims[FS_MAX_RANK] = {1, 1, 1, 1};
  uint32_t rows = 0, cols = 0;
  RowProgP p{};
  std::vector<int32_t> full_in, col_in, rscal_in;   // tensor ids by class (a transposed view of an input: the transpose's result)
  // Transposes that keep the innermost axis only renumber rows.  One applied to a graph input is folded into
  // that input's addressing (the view is then an input of the row program, read with permuted row strides); one
  // that produces a graph output nobody else reads is folded into the store.
  std::vector<int32_t> view_src;     // per tensor: the graph input it is a transposed view of, else -1
  std::vector<int32_t> view_op;      // per tensor: the transpose op that makes the view
  std::vector<int32_t> stored_via;   // per tensor: the transpose op through which it is stored permuted, else -1
  int32_t out_slot[kProgMaxOperands], rout_slot[kProgMaxOperands];
  int n_out = 0, n_rout = 0, n_reductions = 0;
  int n_colsum = 0;                       // column sums over all rows: outputs only, handed out by a fold launch
  int32_t colsum_slot[kProgMaxColSums];   // their fs_execute output slots
  int32_t colsum_dt[kProgMaxColSums];     // the dtype each is handed out in (a fold launch rounds its sums to one dtype)
  std::vector<char> is_colsum;            // per op
  std::vector<char> sum_chain;            // per op: a sum along one leading axis on the way to a column sum (emits nothing)
  int vec_instr = 0, scal_instr = 0, reg_reads = 0, reg_writes = 0, trans = 0;
  std::vector<int> free_regs, free_sregs;
  int acc_holds = -1, sacc_holds = -1;   // roots
  bool planning = true;                  // first pass: only follow the accumulators and note who needs a register
  bool interpretable = true;             // the interpreter has the program's step width (generated kernels have all)

  explicit Compiler(const fs_graph& graph) : g(graph), val(graph.tensors.size()) {}

  int classify(const Tensor& t) const {
    if (t.rank > rank) return V_NONE;
    int64_t d[FS_MAX_RANK];
    for (int k = 0; k < rank; ++k) {
      const int kt = k - (rank - t.rank);
      d[k] = kt >= 0 ? t.dims[kt] : 1;
    }
    bool full = true, rscal = d[rank - 1] == 1, col = d[rank - 1] == dims[rank - 1], stretched = true;
    for (int k = 0; k < rank; ++k) {
      if (d[k] != dims[k]) full = false;
      if (k < rank - 1 && d[k] != dims[k]) rscal = false;
      if (k < rank - 1 && d[k] != 1) col = false;
      if (k < rank - 1 && d[k] != 1 && d[k] != dims[k]) stretched = false;
    }
    if (full) return V_FULL;
    if (rscal) return V_RSCAL;
    if (col) return V_COL;
    // full rows or per-row scalars repeated along some leading axes (see `stretched_rows`)
    if (stretched && d[rank - 1] == dims[rank - 1]) return V_FULL;
    if (stretched && d[rank - 1] == 1) return V_RSCAL;
    return V_NONE;
  }
  // true if `t` has extent 1 on some leading axis where the pattern's row space has more
  bool stretched_rows(const Tensor& t) const {
    const int k0 = rank - t.rank;
    for (int k = 0; k < rank - 1; ++k) {
      const int64_t d = k >= k0 ? t.dims[k - k0] : 1;
      if (d != dims[k]) return true;
    }
    return false;
  }
  void row_strides(const Tensor& T, uint32_t (&ms)[3]) const {
    int64_t acc = 1;
    for (int k = rank - 2; k >= 0; --k) {
      const int kt = k - (rank - T.rank);
      const int64_t d = kt >= 0 ? T.dims[kt] : 1;
      ms[3 - (rank - 1) + k] = d == 1 ? 0u : (uint32_t)acc;
      acc *= d;
    }
  }

  // view = transpose(src, perm), both of the pattern's rank: row of src that holds the view's row, as strides
  // along the pattern's leading axes (axis k of the view is axis perm[k] of src)
  void view_row_strides(const Tensor& src, const int32_t* perm, uint32_t (&ms)[3]) const {
    int64_t stride[FS_MAX_RANK];   // of src, in rows
    int64_t acc = 1;
    for (int k = rank - 2; k >= 0; --k) { stride[k] = acc; acc *= src.dims[k]; }
    for (int k = 0; k < rank - 1; ++k) {
      const int64_t d = src.dims[perm[k]];
      ms[3 - (rank - 1) + k] = (d == 1 && dims[k] != 1) ? 0u : (uint32_t)stride[perm[k]];
    }
  }
  // out = transpose(value, perm): row of out that receives the pattern's row (axis j of the pattern's space is
  // axis k of out with perm[k] == j)
  void store_row_strides(const Tensor& out, const int32_t* perm, uint32_t (&ms)[3]) const {
    int64_t acc = 1;
    for (int k = rank - 2; k >= 0; --k) {
      ms[3 - (rank - 1) + perm[k]] = (uint32_t)acc;
      acc *= out.dims[k];
    }
  }
  bool input_like(int t) const { return g.tensors[t].producer < 0 || view_src[t] >= 0; }

  static bool scalar_shaped(int kind) { return kind == V_RSCAL; }
  int root_of(int tensor) const { return val[tensor].root; }

  int alloc(bool scalar) {
    std::vector<int>& fl = scalar ? free_sregs : free_regs;
    int32_t& n = scalar ? p.n_sregs : p.n_regs;
    if (!fl.empty()) {
      auto it = std::min_element(fl.begin(), fl.end());   // lowest index first keeps the files dense
      const int r = *it;
      fl.erase(it);
      return r;
    }
    return n++;
  }
  void release(int root) {
    Val& v = val[root];
    if (v.reg < 0 || v.input_index >= 0) return;
    (scalar_shaped(v.kind) ? free_sregs : free_regs).push_back(v.reg);
    v.reg = -1;
  }

  // ---- emission ------------------------------------------------------------------------------
  bool push(ProgInstr ins) {
    if (planning) return true;
    if (p.n_instr >= kProgMaxInstr) return false;
    p.instr[p.n_instr++] = ins;
    const bool red = ins.op == PO_RSUM || ins.op == PO_RMAX || ins.op == PO_RSUMSQ;
    if (red) ++n_reductions;
    if (red || (ins.flags & PF_SCALAR) || ins.op == PO_STORE_SCAL) {
      ++scal_instr;
    } else {
      ++vec_instr;
      if (ins.op != PO_STORE && (ins.b_kind == PK_REG || ins.b_kind == PK_COL) &&
          (ins.op <= PO_MAX || ins.op == PO_LOAD)) ++reg_reads;
      if (ins.flags & PF_KEEP) ++reg_writes;
      if (ins.op == PO_DIV || ins.op == PO_RDIV || ins.op == PO_EXP || ins.op == PO_RSQRT) trans += 1;
      if (ins.op == PO_TANH || ins.op == PO_GELU || ins.op == PO_GELU_GRAD || ins.op == PO_SIGMOID) trans += 2;
      if (ins.op == PO_LOG || ins.op == PO_SQRT) trans += 3;   // the quarter-rate instruction plus its range fix-ups
    }
    return true;
  }

  // operand b of an instruction: where root r can be read from, other than "it is the accumulator of
  // its own shape" (that case is PK_ACC / PK_SACC).  In the planning pass a value that is in no
  // accumulator is marked as needing a register.
  bool locate(int r, uint8_t* kind, uint8_t* idx) {
    Val& v = val[r];
    const bool scalar = scalar_shaped(v.kind);
    if (!scalar && v.input_index >= 0) { *kind = PK_COL; *idx = (uint8_t)v.input_index; return true; }
    if (scalar ? sacc_holds == r : acc_holds == r) { *kind = scalar ? PK_SACC : PK_ACC; *idx = 0; return true; }
    if (planning) { v.keep = true; *kind = scalar ? PK_SCAL : PK_REG; *idx = 0; return true; }
    if (v.reg < 0) return false;
    *kind = scalar ? PK_SCAL : PK_REG;
    *idx = (uint8_t)v.reg;
    return true;
  }

  // brings root r into the accumulator of the given shape (full-shaped accumulator may also take a
  // per-row or column value: it is stretched on the way)
  bool load(int r, bool into_scalar) {
    if (into_scalar ? sacc_holds == r : acc_holds == r) return true;
    ProgInstr ld{};
    ld.op = PO_LOAD;
    if (into_scalar) ld.flags = PF_SCALAR;
    if (!locate(r, &ld.b_kind, &ld.b)) return false;
    if (!push(ld)) return false;
    (into_scalar ? sacc_holds : acc_holds) = r;
    return true;
  }

  bool store_output(int t, bool as_full) {
    const Tensor& T = g.tensors[t];
    const int r = root_of(t);
    ProgInstr s{};
    s.aux = (uint8_t)T.store_as;
    if (as_full) {
      if (!planning && n_out >= kProgMaxOperands) return false;
      if (!load(r, false)) return false;
      s.op = PO_STORE;
      if (!planning) {
        if (stored_via[t] >= 0) {
          p.out_perm |= 1u << n_out;
          store_row_strides(T, g.ops[stored_via[t]].perm, p.oms[n_out]);
        }
        s.dst = (uint8_t)n_out;
        out_slot[n_out++] = T.output_slot;
      }
    } else {
      if (!planning && n_rout >= kProgMaxOperands) return false;
      if (!load(r, true)) return false;
      s.op = PO_STORE_SCAL;
      s.flags = PF_SCALAR;
      if (!planning) { s.dst = (uint8_t)n_rout; rout_slot[n_rout++] = T.output_slot; }
    }
    return push(s);
  }

  std::vector<std::vector<int>> reads;
  std::vector<char> is_alias;
  std::vector<int> square_of;   // op j reduces the square of this root (the squaring op itself emits nothing), else -1
  std::vector<char> folded;     // op emits nothing: its work is done by a later instruction

  // One walk over the ops.  planning = true: follow the accumulators, mark values that are read
  // when no accumulator holds them.  planning = false: allocate registers and emit.
  int acc_start = -1;   // full-shaped input the accumulator holds when the walk begins

  bool walk() {
    acc_holds = acc_start;
    sacc_holds = -1;
    const size_t n_ops = g.ops.size();
    for (size_t i = 0; i < n_ops; ++i) {
      const Op& op = g.ops[i];
      const Tensor& out = g.tensors[op.out];
      if (folded[i]) {
        // a transposed view that is itself an output: the pattern's work on it is the move
        if (op.opcode == FS_TRANSPOSE && view_op[op.out] == (int32_t)i && out.output_slot >= 0) {
          if (!store_output(op.out, true)) return false;
          if (!planning && val[op.out].last_read == (int)i) release(op.out);
        }
        continue;
      }
      if (is_colsum[i]) {
        if (!planning && n_colsum >= kProgMaxColSums) return false;
        if (!load(root_of(op.in[0]), false)) return false;
        ProgInstr cs{};
        cs.op = PO_COLSUM;
        cs.b_kind = PK_ACC;
        if (!planning) {
          cs.dst = (uint8_t)n_colsum;
          colsum_dt[n_colsum] = (int32_t)out.store_as;
          colsum_slot[n_colsum++] = out.output_slot;
        }
        if (!push(cs)) return false;
        if (!planning)
          for (int r : reads[i])
            if (val[r].last_read == (int)i) release(r);
      } else if (is_alias[i]) {
        if (out.output_slot >= 0) {
          const bool as_full = op.opcode == FS_BROADCAST || val[op.out].kind != V_RSCAL;
          if (!store_output(op.out, as_full)) return false;
        }
      } else {
        const int ra = square_of[i] >= 0 ? square_of[i] : root_of(op.in[0]), rb = op.n_in > 1 ? root_of(op.in[1]) : -1;
        const bool scalar = scalar_shaped(val[op.out].kind);
        const bool reduce = op.opcode == FS_REDUCE_SUM || op.opcode == FS_REDUCE_MAX || op.opcode == FS_REDUCE_MEAN;
        ProgInstr ins{};
        ins.b_kind = PK_IMM;
        if (scalar && !reduce) ins.flags |= PF_SCALAR;
        int& holds = (scalar && !reduce) ? sacc_holds : acc_holds;   // accumulator the operand(s) go through
        uint8_t fwd = PO_ADD, rev = PO_ADD;
        bool binary = false;
        switch (op.opcode) {
          case FS_ADD: fwd = rev = PO_ADD; binary = true; break;
          case FS_MUL: fwd = rev = PO_MUL; binary = true; break;
          case FS_MAX: fwd = rev = PO_MAX; binary = true; break;
          case FS_SUB: fwd = PO_SUB; rev = PO_RSUB; binary = true; break;
          case FS_DIV: fwd = PO_DIV; rev = PO_RDIV; binary = true; break;
          case FS_SCALE: ins.op = PO_MUL; ins.imm = (float)op.scalar; break;
          case FS_ADD_SCALAR: ins.op = PO_ADD; ins.imm = (float)op.scalar; break;
          case FS_SQUARE: ins.op = PO_SQUARE; break;
          case FS_EXP: ins.op = PO_EXP; break;
          case FS_RSQRT: ins.op = PO_RSQRT; break;
          case FS_TANH: ins.op = PO_TANH; break;
          case FS_GELU_TANH: ins.op = PO_GELU; break;
          case FS_GELU_TANH_GRAD: ins.op = PO_GELU_GRAD; break;
          case FS_LOG: ins.op = PO_LOG; break;
          case FS_SIGMOID: ins.op = PO_SIGMOID; break;
          case FS_RELU: ins.op = PO_RELU; break;
          case FS_ABS: ins.op = PO_ABS; break;
          case FS_SQRT: ins.op = PO_SQRT; break;
          case FS_CONVERT: ins.op = PO_CVT; ins.aux = (uint8_t)op.to_dtype; break;
          case FS_REDUCE_SUM: case FS_REDUCE_MEAN: ins.op = square_of[i] >= 0 ? PO_RSUMSQ : PO_RSUM; break;
          case FS_REDUCE_MAX: ins.op = PO_RMAX; break;
          default: return false;
        }
        if (binary) {
          // the operand already in the accumulator stays there; the other one is b
          if (holds == ra) {
            ins.op = fwd;
            if (!locate(rb, &ins.b_kind, &ins.b)) return false;
          } else if (holds == rb) {
            ins.op = rev;
            if (!locate(ra, &ins.b_kind, &ins.b)) return false;
          } else {
            // neither: bring in the one that can only be read through a register, keep the cheaper source as b
            const bool a_first = !(scalar_shaped(val[ra].kind) && !scalar);   // a per-row value stretches for free as b
            const int first = a_first ? ra : rb, second = a_first ? rb : ra;
            if (!load(first, scalar)) return false;
            ins.op = a_first ? fwd : rev;
            if (!locate(second, &ins.b_kind, &ins.b)) return false;
          }
        } else {
          if (!load(ra, scalar && !reduce)) return false;
        }
        // registers of operands read here for the last time are free for the result
        if (!planning)
          for (int r : reads[i])
            if (val[r].last_read == (int)i) release(r);
        Val& res = val[op.out];
        const bool mean = op.opcode == FS_REDUCE_MEAN;
        if (!planning && res.keep && !mean) {
          res.reg = alloc(scalar);
          ins.flags |= PF_KEEP;
          ins.dst = (uint8_t)res.reg;
        }
        if (!push(ins)) return false;
        if (mean) {
          ProgInstr m{};
          m.op = PO_MUL;
          m.flags = PF_SCALAR;
          m.b_kind = PK_IMM;
          m.imm = (float)(1.0 / (double)cols);
          if (!planning && res.keep) {
            res.reg = alloc(true);
            m.flags |= PF_KEEP;
            m.dst = (uint8_t)res.reg;
          }
          if (!push(m)) return false;
        }
        (scalar ? sacc_holds : acc_holds) = op.out;
        if (out.output_slot >= 0 && !store_output(op.out, !scalar)) return false;
      }
      if (!planning && is_alias[i])
        for (int r : reads[i])
          if (val[r].last_read == (int)i) release(r);
      if (p.n_regs > 250 || p.n_sregs > 250) return false;
    }
    return true;
  }

  std::vector<char> skip_for_anchor;   // per tensor: lives outside the row space (reached through a view or a permuted store)
  std::vector<char> view_fold;         // per op: a transpose folded into an input's addressing

  // The phases of the compilation, in order; each returns false when the pattern does not fit a row program.
  bool run() {
    return fold_transposes() && choose_row_space() && classify_tensors() && classify_ops() && check_outputs() && peepholes() &&
           describe_inputs() && allocate_and_emit();
  }

  bool fold_transposes() {
    // transposes first: which ones fold into a load or a store (any other kind does not fit a row program)
    const size_t n_tensors = g.tensors.size();
    view_src.assign(n_tensors, -1);
    view_op.assign(n_tensors, -1);
    stored_via.assign(n_tensors, -1);
    skip_for_anchor.assign(n_tensors, 0);
    for (size_t i = 0; i < g.ops.size(); ++i) {
      const Op& op = g.ops[i];
      if (op.opcode != FS_TRANSPOSE) continue;
      const Tensor& src = g.tensors[op.in[0]];
      const Tensor& out = g.tensors[op.out];
      if (op.perm[src.rank - 1] != src.rank - 1) return false;   // the innermost axis moves: data crosses rows
      if (src.producer < 0) {
        view_src[op.out] = op.in[0];
        view_op[op.out] = (int32_t)i;
      } else if (out.output_slot >= 0 && out.consumers.empty()) {
        stored_via[op.out] = (int32_t)i;
        skip_for_anchor[op.out] = 1;
      } else {
        return false;
      }
    }
    for (int t : g.inputs) {
      // an input that is only read through transposed views has no place in the row space by itself
      bool only_views = !g.tensors[t].consumers.empty();
      for (int c : g.tensors[t].consumers)
        if (g.ops[c].opcode != FS_TRANSPOSE) only_views = false;
      if (only_views) skip_for_anchor[t] = 1;
    }
    return true;
  }

  bool choose_row_space() {
    const size_t n_tensors = g.tensors.size();
    // anchor = the largest tensor of the row space
    int anchor = -1;
    for (size_t t = 0; t < n_tensors; ++t)
      if (!skip_for_anchor[t] && (anchor < 0 || g.tensors[t].numel() > g.tensors[anchor].numel())) anchor = (int)t;
    if (anchor < 0) return false;
    const Tensor& a = g.tensors[anchor];
    rank = a.rank;
    for (int k = 0; k < rank; ++k) dims[k] = a.dims[k];
    cols = (uint32_t)dims[rank - 1];
    rows = (uint32_t)(a.numel() / cols);
    if (cols < 2) return false;
    return true;
  }

  bool classify_tensors() {
    const size_t n_tensors = g.tensors.size();
    // classes of all tensors; inputs by class
    for (size_t t = 0; t < n_tensors; ++t) {
      const Tensor& T = g.tensors[t];
      if (T.dtype == FS_I32) return false;
      val[t].root = (int)t;
      if (skip_for_anchor[t]) {   // lives outside the row space: reached only through its view / its permuted store
        if (T.rank != rank) return false;
        val[t].kind = V_FULL;
        continue;
      }
      if (view_src[t] >= 0 && T.rank != rank) return false;
      val[t].kind = classify(T);
      if (val[t].kind == V_NONE) return false;
    }
    for (size_t t = 0; t < n_tensors; ++t) {
      if (stored_via[t] < 0) continue;
      // what is stored permuted must be a full-shaped value of the row space, with nothing stretched
      const int src = g.ops[stored_via[t]].in[0];
      if (val[src].kind != V_FULL || classify(g.tensors[src]) != V_FULL || stretched_rows(g.tensors[src])) return false;
    }
    bool narrow = false;   // some vector input is 16 bits wide
    std::vector<int32_t> input_like_tensors;
    for (int t : g.inputs)
      if (!skip_for_anchor[t]) input_like_tensors.push_back(t);
    for (size_t t = 0; t < n_tensors; ++t)
      if (view_src[t] >= 0) input_like_tensors.push_back((int32_t)t);
    for (int t : input_like_tensors) {
      const Tensor& T = g.tensors[t];
      if (view_src[t] >= 0 && val[t].kind != V_FULL) return false;   // a view is addressed by rows
      if (val[t].kind == V_RSCAL) {
        if (rscal_in.size() >= kProgMaxOperands) return false;
        rscal_in.push_back(t);
      } else {
        if (dtype_bytes(T.dtype) == 2) narrow = true;
        std::vector<int32_t>& cls = val[t].kind == V_FULL ? full_in : col_in;
        if (cls.size() >= kProgMaxOperands) return false;
        cls.push_back(t);
      }
      if (T.output_slot >= 0 && view_src[t] < 0) return false;   // an input handed straight to an output is no computation
    }
    // lane geometry by elements: the narrowest vector input still moves in 128-bit accesses where the row length
    // allows it; otherwise 4 elements per step (16-bit inputs then move in 64-bit accesses) or, for rows that are
    // no multiple of 4 elements, single elements (the last two forms exist as generated kernels only)
    p.vec = (narrow && cols % 8 == 0) ? 8 : (cols % 4 == 0 ? 4 : 1);
    interpretable = p.vec == 8 || (p.vec == 4 && !narrow);
    p.rows = rows;
    p.cols = cols;
    return true;
  }

  // A sum over all rows of a pattern with several leading axes is written as a chain: reduce_sum along axis 0, then
  // along axis 1, ... up to the last leading axis, each the only reader of the one before.  Returns the op that ends
  // the chain which op `i` (a reduce_sum along axis 0) starts, or -1.
  int column_sum_chain_end(size_t i) const {
    size_t cur = i;
    for (int ax = 1; ax <= rank - 2; ++ax) {
      const Tensor& t = g.tensors[g.ops[cur].out];
      if (t.output_slot >= 0 || t.consumers.size() != 1) return -1;
      const Op& next = g.ops[t.consumers[0]];
      if (next.opcode != FS_REDUCE_SUM || next.axis != ax) return -1;
      cur = (size_t)t.consumers[0];
    }
    return (int)cur;
  }

  bool classify_ops() {
    // aliases and result classes; which ops read which roots
    const size_t n_ops = g.ops.size();
    sum_chain.assign(n_ops, 0);
    reads.assign(n_ops, {});
    is_alias.assign(n_ops, 0);
    view_fold.assign(n_ops, 0);
    is_colsum.assign(n_ops, 0);
    for (size_t i = 0; i < n_ops; ++i) {
      const Op& op = g.ops[i];
      const Tensor& out = g.tensors[op.out];
      const int ka = val[op.in[0]].kind, kb = op.n_in > 1 ? val[op.in[1]].kind : V_NONE;
      int want = V_NONE;
      switch (op.opcode) {
        case FS_ADD: case FS_SUB: case FS_MUL: case FS_DIV: case FS_MAX:
          if (ka == V_FULL || kb == V_FULL || (ka != kb)) want = V_FULL;
          else want = ka;   // RSCAL x RSCAL or COL x COL
          break;
        case FS_SCALE: case FS_ADD_SCALAR: case FS_SQUARE: case FS_EXP: case FS_RSQRT: case FS_TANH:
        case FS_GELU_TANH: case FS_GELU_TANH_GRAD: case FS_CONVERT:
        case FS_LOG: case FS_SIGMOID: case FS_RELU: case FS_ABS: case FS_SQRT:
          want = ka;
          break;
        case FS_BROADCAST:
          is_alias[i] = 1;
          break;
        case FS_REDUCE_SUM: case FS_REDUCE_MAX: case FS_REDUCE_MEAN: {
          const Tensor& src = g.tensors[op.in[0]];
          if (sum_chain[i] == 1) {   // inside a chain: stands for the value the chain sums
            is_alias[i] = 1;
            val[op.out].kind = V_FULL;
            break;
          }
          if (op.opcode == FS_REDUCE_SUM && op.axis == 0 && src.rank == rank && ka == V_FULL && !stretched_rows(src) && cols % 4 == 0 &&
              sum_chain[i] == 0) {
            const int end = column_sum_chain_end(i);
            const Tensor* last = end >= 0 ? &g.tensors[g.ops[end].out] : nullptr;
            if (last && last->output_slot >= 0 && last->consumers.empty() && last->store_as != FS_I32) {
              // the sum over all rows: every workgroup leaves partial sums, a second launch folds them.  Nothing in the
              // pattern can read it (that would take a grid-wide wait), so it has to be a graph output.
              for (size_t k = i; (int)k != end; k = (size_t)g.tensors[g.ops[k].out].consumers[0]) sum_chain[k] = 1;
              sum_chain[end] = 2;
              if ((int)i != end) {
                is_alias[i] = 1;
                val[op.out].kind = V_FULL;
                break;
              }
            }
          }
          if (sum_chain[i] == 2) {   // the op that completes the sum over all rows
            is_colsum[i] = 1;
            want = V_COL;
            break;
          }
          if (op.axis != src.rank - 1) return false;              // only the row axis stays on chip
          if (ka == V_RSCAL) { want = V_RSCAL; is_alias[i] = 1; }  // reducing one element
          else if (ka == V_FULL) want = V_RSCAL;
          else return false;
          break;
        }
        case FS_TRANSPOSE:
          if (view_src[op.out] >= 0) {   // folded into the input's addressing
            view_fold[i] = 1;
            if (out.output_slot >= 0) reads[i].push_back(op.out);   // stored as it is read
            continue;
          }
          if (stored_via[op.out] != (int32_t)i) return false;
          is_alias[i] = 1;                                              // folded into the store
          break;
        default:
          return false;
      }
      if (is_alias[i]) {
        if (op.opcode == FS_BROADCAST) {
          // stretching may only go toward the pattern's row space; the result keeps the source's class
          // (readers stretch it on the fly)
          if (val[op.out].kind != V_FULL && val[op.out].kind != ka) return false;
          if (out.output_slot >= 0 && classify(out) != V_FULL) return false;
          val[op.out].kind = ka;
        }
        val[op.out].root = val[op.in[0]].root;
        if (out.output_slot >= 0) reads[i].push_back(val[op.out].root);   // its store reads the root
      } else {
        if (val[op.out].kind != want) return false;
        reads[i].push_back(val[op.in[0]].root);
        if (op.n_in > 1) reads[i].push_back(val[op.in[1]].root);
      }
    }
    return true;
  }

  bool check_outputs() {
    for (int t : g.outputs) {
      if (g.tensors[t].producer < 0) return false;
      if (stored_via[t] >= 0) continue;   // a permutation of the row space: every row is written once
      if (is_colsum[g.tensors[t].producer]) continue;   // one value per column, left by the fold launch
      const int shape = classify(g.tensors[t]);
      if (shape != V_FULL && shape != V_RSCAL) return false;   // a per-column value has no row to be stored to
      if (stretched_rows(g.tensors[t])) return false;   // an output must own every row it is stored to
    }
    return true;
  }

  bool peepholes() {
    const size_t n_ops = g.ops.size();
    // peepholes.  (1) square feeding only a row sum / mean: the reduction squares on the fly, so the
    // accumulator keeps the un-squared value.  (2) a convert whose only reader is the store of the same
    // dtype: the store rounds anyway.
    std::vector<int> n_reads(g.tensors.size(), 0);
    for (size_t i = 0; i < n_ops; ++i)
      for (int r : reads[i]) ++n_reads[r];
    square_of.assign(n_ops, -1);
    folded.assign(n_ops, 0);
    for (size_t i = 0; i < n_ops; ++i)
      if (view_fold[i]) folded[i] = 1;
    for (size_t i = 0; i + 1 < n_ops; ++i) {
      const Op& op = g.ops[i];
      if (op.opcode != FS_SQUARE || is_alias[i] || val[op.out].kind != V_FULL) continue;
      if (g.tensors[op.out].output_slot >= 0 || n_reads[op.out] != 1) continue;
      size_t j = i + 1;
      while (j < n_ops && (is_alias[j] && reads[j].empty())) ++j;
      if (j >= n_ops || is_alias[j]) continue;
      const Op& red = g.ops[j];
      if ((red.opcode != FS_REDUCE_SUM && red.opcode != FS_REDUCE_MEAN) || val[red.in[0]].root != op.out || is_colsum[j]) continue;
      folded[i] = 1;
      square_of[j] = val[op.in[0]].root;
      reads[i].clear();
      reads[j].assign(1, square_of[j]);
    }
    for (size_t i = 0; i < n_ops; ++i) {
      const Op& op = g.ops[i];
      const Tensor& out = g.tensors[op.out];
      if (op.opcode != FS_CONVERT || is_alias[i] || val[op.out].kind != V_FULL) continue;
      if (out.output_slot < 0 || n_reads[op.out] != 0 || out.store_as != op.to_dtype) continue;
      is_alias[i] = 1;
      val[op.out].root = val[op.in[0]].root;
      reads[i].assign(1, val[op.out].root);
    }
    for (size_t i = 0; i < n_ops; ++i)
      for (int r : reads[i]) val[r].last_read = (int)i;
    return true;
  }

  bool describe_inputs() {
    // inputs: column vectors sit in the shared column file, the others are parked in registers
    p.n_full = (int32_t)full_in.size();
    p.n_col = (int32_t)col_in.size();
    p.n_rscal = (int32_t)rscal_in.size();
    for (size_t i = 0; i < col_in.size(); ++i) {
      val[col_in[i]].input_index = (int)i;
      p.col_dt[i] = (uint8_t)g.tensors[col_in[i]].dtype;
    }
    for (size_t i = 0; i < full_in.size(); ++i) p.full_dt[i] = (uint8_t)g.tensors[full_in[i]].dtype;
    // leading axes of the row space, collapsed to three; inputs stretched along some of them get row strides
    {
      uint32_t od[3] = {1, 1, 1};
      for (int k = 0; k < rank - 1; ++k) od[3 - (rank - 1) + k] = (uint32_t)dims[k];
      for (int k = 0; k < 3; ++k) {
        p.od[k] = make_fastdiv(od[k]);
        if (p.od[k].d == 0) return false;
      }
      for (size_t i = 0; i < full_in.size(); ++i) {
        const Tensor& T = g.tensors[full_in[i]];
        if (view_src[full_in[i]] >= 0) {   // rows renumbered by the folded transpose
          p.full_bcast |= 1u << i;
          view_row_strides(g.tensors[view_src[full_in[i]]], g.ops[view_op[full_in[i]]].perm, p.ms[i]);
          continue;
        }
        if (!stretched_rows(T)) continue;
        p.full_bcast |= 1u << i;
        row_strides(T, p.ms[i]);
      }
      for (size_t i = 0; i < rscal_in.size(); ++i) {
        const Tensor& T = g.tensors[rscal_in[i]];
        if (!stretched_rows(T)) continue;
        p.rscal_bcast |= 1u << i;
        row_strides(T, p.rms[i]);
      }
    }
    return true;
  }

  bool allocate_and_emit() {
    const size_t n_ops = g.ops.size();
    // the first op's full-shaped input operand is handed over in the accumulator by the prologue;
    // it is parked in a register as well only if something reads it after the accumulator moved on
    p.acc_input = -1;
    for (size_t i = 0; i < n_ops && acc_start < 0; ++i) {
      if (reads[i].empty()) continue;
      for (int r : reads[i])
        if (acc_start < 0 && val[r].kind == V_FULL && input_like(r)) acc_start = r;
      break;
    }
    planning = true;
    if (!walk()) return false;
    planning = false;
    for (size_t i = 0; i < full_in.size(); ++i) {
      const int t = full_in[i];
      if (t == acc_start) p.acc_input = (int32_t)i;
      if (t == acc_start && !val[t].keep) { p.full_reg[i] = 255; continue; }
      p.full_reg[i] = (uint8_t)(val[t].reg = alloc(false));
    }
    for (size_t i = 0; i < rscal_in.size(); ++i) {
      p.rscal_sreg[i] = (uint8_t)(val[rscal_in[i]].reg = alloc(true));
      p.rscal_dt[i] = (uint8_t)g.tensors[rscal_in[i]].dtype;
    }
    for (int t : g.inputs)
      if (val[t].last_read < 0) release(t);   // declared but unread
    if (!walk()) return false;
    if ((int)full_in.size() > kProgMaxInterpretedFull) interpretable = false;
    p.n_colsum = n_colsum;
    p.rows_per_group = 1;
    p.col_tiles = 1;
    p.col_chunks = 1;
    p.col_kept = 0;
    if (n_colsum > 0) interpretable = false;
    return n_out + n_rout + n_colsum == (int)g.outputs.size();
  }
};

// ---- launch shapes and candidates ------------------------------------------------------------------------

// How a row program is laid over the device: L lanes of a wavefront (or the whole 256-thread workgroup) per row, K
// steps of `vec` elements per lane; generated kernels with column sums also R rows per lane group, one after the
// other, and CT column tiles.
struct Shape {
  uint32_t L;
  int K;
  bool block;
  bool generated;
  uint32_t R = 1, CT = 1;
  uint32_t NC = 1;   // > 1: the row is worked through in NC chunks of L * K steps (rows beyond any workgroup's registers)
  uint32_t kept = 0; // of those, the first `kept` stay in registers in storage form after the first pass
};

// Step widths to offer.  A pattern whose 16-bit vector inputs ask for 8 elements per step may also move float32
// rows (an input, or an output stored as float32): those take two 128-bit accesses per step, 32 bytes apart per
// lane, which the memory system likes less than one; 4 elements per step turns that around (float32 in one
// access, the 16-bit operands in 64-bit ones).  Both are offered then, the narrower one as generated kernels.
std::vector<int> step_widths(const RowProgP& base) {
  bool moves_f32_rows = false;
  for (int i = 0; i < base.n_full; ++i) moves_f32_rows = moves_f32_rows || base.full_dt[i] == DT_F32;
  for (int i = 0; i < base.n_instr; ++i) moves_f32_rows = moves_f32_rows || (base.instr[i].op == PO_STORE && base.instr[i].aux == DT_F32);
  std::vector<int> widths(1, base.vec);
  if (base.vec == 8 && moves_f32_rows && codegen_enabled()) widths.push_back(4);
  return widths;
}

// Column sums: a workgroup's lane groups work through R rows each and leave one row of partial sums, so R trades
// extra traffic (2 x workgroups x columns x 4 bytes) against workgroups to fill the chip with.  Every generated
// shape is offered with R = 1, 2, 4, ... while at least one workgroup per compute unit remains.
std::vector<Shape> with_rows_per_group(const std::vector<Shape>& shapes, uint32_t rows) {
  std::vector<Shape> out;
  for (const Shape& sh : shapes) {
    if (!sh.generated) continue;
    const uint32_t rows_per_wg = sh.block ? 1 : 256 / sh.L;
    auto workgroups = [&](uint32_t R) { return (rows + (uint64_t)rows_per_wg * R - 1) / ((uint64_t)rows_per_wg * R) * sh.CT; };
    std::vector<uint32_t> offered;
    bool some_moderate = false;
    for (uint32_t R : {1u, 2u, 4u, 8u, 16u, 32u, 64u}) {
      if (R > 1 && workgroups(R) < 256) break;
      offered.push_back(R);
      some_moderate = some_moderate || workgroups(R) <= 8192;
    }
    for (uint32_t R : offered) {
      // thousands of workgroups more than the chip holds only multiply the partial sums: not offered when a
      // larger R brings the count down
      if (some_moderate && workgroups(R) > 8192) continue;
      Shape t = sh;
      t.R = R;
      out.push_back(t);
    }
  }
  return out;
}

std::vector<Shape> enumerate_shapes(const Compiler& c, int vec, bool interpretable) {
  const uint32_t nvec = c.p.cols / vec;
  std::vector<Shape> shapes;
  if (interpretable) {
    for (int K : {1, 2, 4}) {
      uint32_t L = 1;
      while (L * (uint32_t)K < nvec) L <<= 1;
      if (L <= 64 && !(K > 1 && (uint64_t)L * K >= 2ull * nvec)) shapes.push_back({L, K, false, false});
    }
    if (c.n_reductions <= kProgMaxReductions)
      for (int K : {1, 2, 4})
        if (256ull * K >= nvec && 64ull * K < nvec) shapes.push_back({256, K, true, false});   // rows a wavefront cannot hold at this K
  }
  if (!codegen_enabled()) return shapes;
  // generated kernels (listed after the interpreted ones, whose indices stay): any number of steps per lane up to
  // 8 (32 single-element steps), so a row can fill its lanes exactly (768 floats: 32 lanes x 6 vectors)
  const uint32_t max_k = vec == 1 ? 32 : 8;
  for (uint32_t L = 1; L <= 64; L <<= 1) {
    const uint32_t K = (nvec + L - 1) / L;
    if (K >= 1 && K <= max_k && (L == 1 || (uint64_t)(L / 2) * K < nvec)) shapes.push_back({L, (int)K, false, true});
  }
  // long rows: a workgroup per row, of 256 threads, or of 512 / 1024 when that takes steps off every lane
  for (uint32_t T : {256u, 512u, 1024u}) {
    const uint32_t KB = (nvec + T - 1) / T;
    // (with column sums a workgroup walks many rows, so few workgroups are resident: there a row may also take exactly
    // one step of 512 or 1024 lanes, which puts more wavefronts on a compute unit)
    if (KB <= max_k && 64ull * 2 < nvec && (T == 256 || nvec > (uint64_t)T || (c.n_colsum > 0 && nvec == (uint64_t)T)))
      shapes.push_back({T, (int)KB, true, true});
  }
  // rows beyond 1024 threads x max_k steps: chunks of a workgroup's worth of steps, a pass per row reduction
  // (also offered, on 1024 threads, to shorter rows whose pattern keeps more values than a lane has registers for).
  // Patterns with reductions are offered a second form of each wide shape in which as many chunks as the register
  // file has room for stay in registers in storage form after the first pass.
  if (nvec > 256ull * max_k && c.n_colsum == 0)
    for (uint32_t T : {256u, 512u, 1024u})
      for (uint32_t K : {max_k / 4, max_k / 2, max_k}) {
        Shape t{T, (int)K, true, true};
        t.NC = (nvec + T * K - 1) / (T * K);
        if (t.NC < 2 || t.NC > 4096) continue;
        const bool plain = nvec <= 1024ull * max_k ? (T == 1024 && K < max_k) : K != max_k / 4;
        if (plain) shapes.push_back(t);
        if (c.n_reductions == 0 || T == 256) continue;
        int regs_per_chunk = 0;   // registers a lane needs to keep one chunk of every row operand
        for (int i = 0; i < c.p.n_full; ++i) regs_per_chunk += (int)K * ((vec * dtype_bytes(c.p.full_dt[i]) + 3) / 4);
        const int body = 24 + (int)K * vec * (c.p.n_regs + 1 + (c.p.n_col > 0 ? 1 : 0)) + 2 * (int)K * c.p.n_full;
        const int room = 512 / (int)(T / 256) - body - 8;
        if (regs_per_chunk == 0 || room < regs_per_chunk) continue;
        t.kept = std::min<uint32_t>(t.NC, (uint32_t)(room / regs_per_chunk));
        if (t.NC - t.kept <= 64) shapes.push_back(t);   // the kept chunks are written out one by one: keep the source short
      }
  if (c.n_colsum == 0) return shapes;
  // Without row reductions nothing ties the columns of a row together: a workgroup may take one tile of 64 or 128
  // vectors, so a lane keeps one or two vectors per value whatever the row length.
  if (c.n_reductions == 0 && c.n_rout == 0)
    for (int K : {1, 2}) {
      const uint32_t tile_vecs = 64u * K;
      if (nvec % tile_vecs == 0 && nvec / tile_vecs > 1 && nvec / tile_vecs <= 4096) {
        Shape t{64, K, false, true};
        t.CT = nvec / tile_vecs;
        shapes.push_back(t);
      }
    }
  return with_rows_per_group(shapes, c.p.rows);
}

// The launch of the program in shape `s` (interpreted form), with its buffer bindings.
void fill_launch(const fs_graph& g, const Compiler& c, int vec, const Shape& s, int64_t lds, Launch* l) {
  l->kernel = K_ROW_PROGRAM;
  RowProgP q = c.p;
  q.vec = vec;
  q.lanes_per_row = (int32_t)s.L;
  int lg = 0;
  while ((1u << lg) < s.L) ++lg;
  q.lanes_log2 = lg;
  q.vecs_per_lane = s.K;
  q.rows_per_group = (int32_t)s.R;
  q.col_tiles = (int32_t)s.CT;
  q.col_chunks = (int32_t)s.NC;
  q.col_kept = (int32_t)s.kept;
  l->args.u.prog = q;
  auto in_ref = [&](int32_t t) {   // a transposed view binds the buffer of the input it views
    BufRef r;
    r.kind = BUF_INPUT;
    r.slot = g.tensors[c.view_src[t] >= 0 ? c.view_src[t] : t].input_slot;
    return r;
  };
  for (size_t i = 0; i < c.full_in.size(); ++i) l->ptr[kSlotFull + i] = in_ref(c.full_in[i]);
  for (size_t i = 0; i < c.col_in.size(); ++i) l->ptr[kSlotCol + i] = in_ref(c.col_in[i]);
  for (size_t i = 0; i < c.rscal_in.size(); ++i) l->ptr[kSlotRscal + i] = in_ref(c.rscal_in[i]);
  for (int i = 0; i < c.n_out; ++i) { l->ptr[kSlotOut + i].kind = BUF_OUTPUT; l->ptr[kSlotOut + i].slot = c.out_slot[i]; }
  for (int i = 0; i < c.n_rout; ++i) { l->ptr[kSlotRout + i].kind = BUF_OUTPUT; l->ptr[kSlotRout + i].slot = c.rout_slot[i]; }
  const uint32_t rows_per_block = (s.block ? 1 : 256 / s.L) * s.R;
  l->shape.block[0] = s.block ? s.L : 256;
  l->shape.grid[0] = (c.p.rows + rows_per_block - 1) / rows_per_block * s.CT;
  l->shape.lds_bytes = (uint32_t)lds;
}

// What the interpreter does per element and per wavefront in shape `s`.
KernelCost interpreted_cost(const Compiler& c, int vec, const Shape& s, int64_t lds, int64_t bytes_min, uint32_t grid) {
  const RowProgP& base = c.p;
  const int kv = s.K * vec;
  const uint32_t nvec = base.cols / vec;
  const double n = (double)base.rows * base.cols;
  double in_bytes_per_elem = 0, col_bytes_per_elem = 0, narrowest = 4.0;
  for (int i = 0; i < base.n_full; ++i) {
    in_bytes_per_elem += dtype_bytes(base.full_dt[i]);
    narrowest = std::min(narrowest, (double)dtype_bytes(base.full_dt[i]));
  }
  for (int i = 0; i < base.n_col; ++i) col_bytes_per_elem += dtype_bytes(base.col_dt[i]);
  KernelCost kc;
  kc.hbm_bytes = (double)bytes_min;
  if (vec == 8) {
    // float32 rows under 8-element steps move as two 128-bit accesses 32 bytes apart per lane (measured: about a
    // quarter more time for those bytes than one access per lane takes)
    int f32_rows = 0;
    for (int i = 0; i < base.n_full; ++i) f32_rows += base.full_dt[i] == DT_F32 && !((base.full_bcast >> i) & 1u);
    for (int i = 0; i < base.n_instr; ++i) f32_rows += base.instr[i].op == PO_STORE && base.instr[i].aux == DT_F32;
    kc.hbm_bytes += 0.25 * 4.0 * n * f32_rows;
  }
  kc.cache_bytes = col_bytes_per_elem * n;
  kc.elems = n;
  // per element: the op itself plus operand / result moves; per instruction and wave: ~40 scalar-side cycles of dispatch
  const double dispatch = 40.0 * base.n_instr / (64.0 * kv) / 4.0;
  kc.valu_per_elem = 2.5 * c.vec_instr + dispatch + 2.0 * base.n_full;
  kc.trans_per_elem = c.trans;
  kc.lds_traffic_bytes = n * 4.0 * (c.reg_reads + c.reg_writes + base.n_full);
  kc.waves_per_block = s.block ? (int32_t)(s.L / 64) : 4;
  kc.waves = (double)grid * kc.waves_per_block;
  kc.bytes_in_flight_per_lane = (vec == 1 ? (double)in_bytes_per_elem : std::max(16.0, (double)vec * in_bytes_per_elem)) * s.K;
  kc.vgpr_estimate = 40 + 3 * kv + 4 * s.K * (base.n_full <= 1 ? 1 : (base.n_full <= 2 ? 2 : 4));
  int steps = 0;
  for (uint32_t t = 1; t < std::min<uint32_t>(s.L, 64); t <<= 1) ++steps;
  kc.xlane_steps = steps * c.n_reductions;
  kc.barriers = s.block ? c.n_reductions : 0;
  kc.lds_bytes_per_block = (int32_t)lds;
  kc.lane_utilisation = (double)(nvec / s.CT) / ((double)s.L * s.K);
  // contiguous bytes the lanes of one row touch per access of the narrowest input
  const double run = (double)std::min<uint32_t>(s.L, 64) * vec * narrowest;
  kc.access_run_bytes = run >= 128.0 ? 0.0 : run;
  kc.preamble_instr = 60;
  return kc;
}

// Turns an interpreted candidate into the generated one of the same shape: the same program as straight-line
// code of its own, every value in registers, no dispatch, no LDS files.
void make_generated(const Compiler& c, int vec, const Shape& s, Candidate* cand) {
  const RowProgP& base = c.p;
  const int kv = s.K * vec;
  Launch& gl = cand->launches.back();
  gl.kernel = K_ROW_GENERATED;
  gl.shape.lds_bytes = 0;
  const int32_t slots = s.block ? (int32_t)(s.L / 64) * 4 * c.n_reductions : 0;
  cand->info.lds_bytes = slots;
  snprintf(cand->info.pattern, sizeof cand->info.pattern, "row_generated");
  snprintf(cand->info.kernel, sizeof cand->info.kernel, "row_generated<v%d,K%d,L%u,I%d,R%d>", vec, s.K, s.L, base.n_instr, base.n_regs);
  KernelCost& gc = cand->cost;
  gc.valu_per_elem = 1.0 * c.vec_instr + 1.0 * base.n_full + 1.0 * c.n_out;
  gc.lds_traffic_bytes = 0;
  gc.lds_bytes_per_block = slots;
  gc.vgpr_estimate = 24 + kv * (base.n_regs + 1 + (base.n_col > 0 ? 1 : 0)) + 2 * s.K * base.n_full;
  gc.preamble_instr = 40;
  // a lane's own instruction stream between its loads landing and its stores leaving: the first and the last
  // wavefronts of the launch run it with the memory system idle, so long per-lane chains (many vectors per
  // lane) cost time that more, shorter wavefronts would have overlapped
  const DeviceModel& d = device();
  gc.serial_tail_s = 1.5 * kv * (gc.valu_per_elem * d.cycles_valu + gc.trans_per_elem * d.cycles_trans) / d.clock_hz;
  if (s.NC > 1) {
    // a pass over the row per reduction re-reads the operands (counted as device-memory traffic: the rows in flight
    // are larger than the caches in general) and repeats the arithmetic before its reduction
    if (s.kept > 0)
      snprintf(cand->info.kernel, sizeof cand->info.kernel, "row_generated<v%d,K%d,L%u,I%d,R%d,chunks%u,kept%u>", vec, s.K, s.L, base.n_instr,
               base.n_regs, s.NC, s.kept);
    else
      snprintf(cand->info.kernel, sizeof cand->info.kernel, "row_generated<v%d,K%d,L%u,I%d,R%d,chunks%u>", vec, s.K, s.L, base.n_instr,
               base.n_regs, s.NC);
    double in_bytes = 0;
    int regs_per_chunk = 0;
    for (int i = 0; i < base.n_full; ++i) {
      if (!((base.full_bcast >> i) & 1u)) in_bytes += (double)dtype_bytes(base.full_dt[i]) * base.rows * base.cols;
      regs_per_chunk += s.K * ((vec * dtype_bytes(base.full_dt[i]) + 3) / 4);
    }
    in_bytes *= 1.0 - (double)s.kept / s.NC;   // chunks kept in registers are not read again
    gc.vgpr_estimate += regs_per_chunk * (int)s.kept;
    // ... unless the rows the resident workgroups are working on fit the memory-side cache (with room for the
    // outputs passing through): wide workgroups keep fewer rows in flight
    const double wgs_per_cu = std::max(1.0, std::floor(2048.0 / s.L));
    const double rows_in_flight_bytes = d.n_cu * wgs_per_cu * in_bytes / base.rows;
    // (every other pass walks the row backwards, so even a set of rows larger than the cache finds the chunks read last;
    // measured on 128256-column rows: a re-read costs 0.35 to 0.5 of a pass from device memory while the rows in flight
    // fit, 0.55 to 0.65 at two to four times the cache)
    const double fit = std::min(1.0, 0.6 * d.last_level_cache_bytes / std::max(1.0, rows_in_flight_bytes));
    const double reread = d.last_level_reread + (0.8 - d.last_level_reread) * (1.0 - fit);
    // a row maximum that only keeps the exponentials of a sum in range shares its pass with that sum
    const int extra_passes = c.n_reductions - online_reduction_pairs(base, nullptr);
    gc.hbm_bytes += in_bytes * extra_passes * reread;
    cand->info.bytes_moved_model += (int64_t)(in_bytes * extra_passes);
    gc.valu_per_elem *= 1.0 + 0.5 * extra_passes;
    gc.trans_per_elem *= 1.0 + 0.5 * c.n_reductions;
    gc.lane_utilisation = (double)(base.cols / vec) / ((double)s.L * s.K * s.NC);
    gc.serial_tail_s += d.mem_latency_s * c.n_reductions;
    // a first pass that gathers maximum and sum together issues the loads of every kept chunk before it works on the first
    if (s.kept > 0 && extra_passes < c.n_reductions) gc.bytes_in_flight_per_lane *= (double)s.kept;
  }
}

// Column sums of a generated candidate: partial sums of every workgroup through the workspace, folded by a second
// launch (one hand-off through device memory: the GLOBAL scheme).
void add_column_sums(const Compiler& c, int vec, const Shape& s, int64_t bytes_min, Candidate* cand) {
  const RowProgP& base = c.p;
  const int kv = s.K * vec;
  const DeviceModel& d = device();
  Launch& ml = cand->launches.back();
  const uint32_t n_wg = ml.shape.grid[0] / s.CT;   // one row of partial sums per row block (its column tiles share the row)
  const uint32_t width = (uint32_t)c.n_colsum * base.cols;
  ml.ptr[kSlotWs].kind = BUF_WORKSPACE;
  ml.ptr[kSlotWs].offset = 0;
  cand->info.lds_bytes += s.block ? 0 : c.n_colsum * 4 * (int32_t)(s.L * kv) * 4;
  // a fold hands out two neighbouring sums of one dtype (or one sum) from its slice of the partial rows; the folds
  // are kept as one record each and issued together as one launch
  for (int first = 0, here = 0; first < c.n_colsum; first += here) {
    here = (first + 1 < c.n_colsum && c.colsum_dt[first] == c.colsum_dt[first + 1]) ? 2 : 1;
    cand->launches.emplace_back();
    Launch& f = cand->launches.back();
    make_fold_launch(&f, n_wg, (uint32_t)here * base.cols, base.cols, width, c.colsum_dt[first]);
    f.ptr[0].kind = BUF_WORKSPACE;
    f.ptr[0].offset = (int64_t)first * base.cols * 4;
    for (int i = 0; i < here; ++i) {
      f.ptr[1 + i].kind = BUF_OUTPUT;
      f.ptr[1 + i].slot = c.colsum_slot[first + i];
    }
  }
  cand->info.scheme = FS_SCHEME_GLOBAL;
  cand->info.n_kernels = 2;   // the pattern's kernel, and its folds as one launch
  cand->info.workspace_bytes = (int64_t)n_wg * width * 4;
  cand->info.bytes_moved_model = bytes_min + 2 * cand->info.workspace_bytes;
  if (s.CT > 1)
    snprintf(cand->info.kernel, sizeof cand->info.kernel, "row_generated<v%d,K%d,L%u,I%d,R%d,rows%u,tiles%u>+colfold", vec, s.K, s.L,
             base.n_instr, base.n_regs, s.R, s.CT);
  else
    snprintf(cand->info.kernel, sizeof cand->info.kernel, "row_generated<v%d,K%d,L%u,I%d,R%d,rows%u>+colfold", vec, s.K, s.L, base.n_instr,
             base.n_regs, s.R);
  KernelCost& gc = cand->cost;
  gc.hbm_bytes += 2.0 * (double)cand->info.workspace_bytes;
  gc.vgpr_estimate += kv * c.n_colsum;
  gc.rows_per_wave_loop = s.R;
  if (s.R > 1) {   // software-pipelined: only the first row's load latency is exposed
    gc.dep_phases = 0;
    gc.serial_tail_s += d.mem_latency_s;
    gc.bytes_in_flight_per_lane *= 2.0;   // this row's and the next row's loads
  }
  gc.lds_bytes_per_block = cand->info.lds_bytes;
  gc.barriers = 1;
  gc.serial_tail_s += (d.mem_latency_s + 0.5 * d.launch_s + d.mem_latency_s * std::ceil(n_wg / 64.0 / 8.0) * 0.5) * 1.0;
}

// One candidate: the program in shape `s`, interpreted or generated.  false: the shape does not fit (the
// interpreter's register files beyond its LDS budget, a generated kernel beyond the register file).
bool make_candidate(const fs_graph& g, const Compiler& c, int vec, const Shape& s, int64_t bytes_min, Candidate* cand) {
  const RowProgP& base = c.p;
  const int kv = s.K * vec;
  const int64_t lds = (int64_t)base.n_regs * kv * 4 * 256 + (int64_t)base.n_col * base.cols * 4 + (int64_t)base.n_sregs * 1024 +
                      kProgMaxReductions * 16;
  if (!s.generated && lds > kProgMaxLdsBytes) return false;
  memset(&cand->info, 0, sizeof cand->info);
  cand->info.scheme = s.block ? FS_SCHEME_LDS : (s.L == 1 ? FS_SCHEME_LOCAL : FS_SCHEME_WAVE);
  cand->info.n_kernels = 1;
  cand->info.bytes_min = bytes_min;
  cand->info.bytes_moved_model = bytes_min;
  snprintf(cand->info.pattern, sizeof cand->info.pattern, "row_program");
  cand->launches.emplace_back();
  Launch& l = cand->launches.back();
  fill_launch(g, c, vec, s, lds, &l);
  cand->info.lanes_per_row = (int32_t)s.L;
  cand->info.vecs_per_lane = s.K;
  cand->info.rows_per_block = (int32_t)((s.block ? 1 : 256 / s.L) * s.R);
  cand->info.lds_bytes = (int32_t)lds;
  for (int k = 0; k < 3; ++k) { cand->info.block[k] = (int32_t)l.shape.block[k]; cand->info.grid[k] = (int32_t)l.shape.grid[k]; }
  snprintf(cand->info.kernel, sizeof cand->info.kernel, "row_program<v%d,K%d,L%u,I%d,R%d>", vec, s.K, s.L, base.n_instr, base.n_regs);
  cand->cost = interpreted_cost(c, vec, s, lds, bytes_min, l.shape.grid[0]);
  cand->fallback = !s.generated && codegen_enabled();
  if (!s.generated) return true;
  make_generated(c, vec, s, cand);
  if (c.n_colsum > 0) add_column_sums(c, vec, s, bytes_min, cand);
  // more would not fit the register file without spilling: 512 registers per SIMD lane are shared by the workgroup's
  // wavefronts on that SIMD (4 of a 1024-thread workgroup, 2 of a 512-thread one)
  const int budget = s.block && s.L > 256 ? 512 / (int)(s.L / 256) : 256;
  return cand->cost.vgpr_estimate <= budget;
}

}  // namespace

bool build_row_program(const fs_graph& g, std::vector<Candidate>* out) {
  Compiler c(g);
  if (!c.run()) return false;
  const int64_t bytes_min = graph_bytes_min(g);
  for (int vec : step_widths(c.p)) {
    const bool interpretable = c.interpretable && vec == c.p.vec;
    for (const Shape& s : enumerate_shapes(c, vec, interpretable)) {
      Candidate cand;
      if (make_candidate(g, c, vec, s, bytes_min, &cand)) out->push_back(cand);
    }
  }
  return !out->empty();
}

}  // namespace fs
