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
// Each op's result goes to the accumulator of its shape; it is also written to a register
// only if some reader comes after the accumulator has been overwritten (look-ahead over
// the op list).  Registers are reused once their last reader has run.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "fs_internal.hpp"

namespace fs {
namespace {

enum ValKind : int { V_NONE = 0, V_FULL, V_RSCAL, V_COL };

struct Val {
  int kind = V_NONE;
  int root = -1;        // tensor whose storage this value shares (itself unless an alias)
  int reg = -1;         // register index in the file of its shape, -1 = none
  int input_index = -1; // column input: its position in the shared column file
  int last_read = -1;   // index of the last op that reads the root
  bool keep = false;
};

struct Compiler {
  const fs_graph& g;
  std::vector<Val> val;
  int rank = 0;
  int64_t dims[FS_MAX_RANK] = {1, 1, 1, 1};
  uint32_t rows = 0, cols = 0;
  RowProgP p{};
  std::vector<int32_t> full_in, col_in, rscal_in;   // tensor ids by class
  int32_t out_slot[kProgMaxOperands], rout_slot[kProgMaxOperands];
  int n_out = 0, n_rout = 0, n_reductions = 0;
  int vec_instr = 0, scal_instr = 0, reg_reads = 0, reg_writes = 0, trans = 0;
  std::vector<int> free_regs, free_sregs;
  int acc_holds = -1, sacc_holds = -1;

  explicit Compiler(const fs_graph& graph) : g(graph), val(graph.tensors.size()) {}

  int classify(const Tensor& t) const {
    if (t.rank > rank) return V_NONE;
    int64_t d[FS_MAX_RANK];
    for (int k = 0; k < rank; ++k) {
      const int kt = k - (rank - t.rank);
      d[k] = kt >= 0 ? t.dims[kt] : 1;
    }
    bool full = true, rscal = d[rank - 1] == 1, col = d[rank - 1] == dims[rank - 1];
    for (int k = 0; k < rank; ++k) {
      if (d[k] != dims[k]) full = false;
      if (k < rank - 1 && d[k] != dims[k]) rscal = false;
      if (k < rank - 1 && d[k] != 1) col = false;
    }
    if (full) return V_FULL;
    if (rscal) return V_RSCAL;
    if (col) return V_COL;
    return V_NONE;
  }

  bool is_scalar_shaped(int kind) const { return kind == V_RSCAL; }

  int alloc(bool scalar) {
    std::vector<int>& fl = scalar ? free_sregs : free_regs;
    int32_t& n = scalar ? p.n_sregs : p.n_regs;
    if (!fl.empty()) {
      // lowest index first keeps the files dense
      auto it = std::min_element(fl.begin(), fl.end());
      const int r = *it;
      fl.erase(it);
      return r;
    }
    return n++;
  }
  void release(int root) {
    Val& v = val[root];
    if (v.reg < 0) return;
    (is_scalar_shaped(v.kind) ? free_sregs : free_regs).push_back(v.reg);
    v.reg = -1;
  }

  bool operand(int tensor, uint8_t* kind, uint8_t* idx) const {
    const Val& v = val[val[tensor].root];
    if (is_scalar_shaped(v.kind)) {
      if (sacc_holds == v.root) { *kind = PK_SACC; *idx = 0; return true; }
      if (v.reg < 0) return false;
      *kind = PK_SCAL;
    } else {
      if (v.input_index >= 0) {
        *kind = PK_COL;
        *idx = (uint8_t)v.input_index;
        return true;
      }
      if (acc_holds == v.root) { *kind = PK_ACC; *idx = 0; return true; }
      if (v.reg < 0) return false;
      *kind = PK_REG;
    }
    *idx = (uint8_t)v.reg;
    return true;
  }

  bool emit(const ProgInstr& ins) {
    if (p.n_instr >= kProgMaxInstr) return false;
    p.instr[p.n_instr++] = ins;
    if (ins.op == PO_RSUM || ins.op == PO_RMAX) {
      ++n_reductions;
      ++scal_instr;
    } else if (ins.flags & PF_SCALAR) {
      ++scal_instr;
    } else {
      ++vec_instr;
    }
    if (!(ins.flags & PF_SCALAR) || ins.op == PO_RSUM || ins.op == PO_RMAX) {
      if (ins.a_kind == PK_REG || ins.a_kind == PK_COL) ++reg_reads;
      if (ins.op <= PO_MAX && (ins.b_kind == PK_REG || ins.b_kind == PK_COL)) ++reg_reads;
      if ((ins.flags & PF_KEEP) && !(ins.op == PO_RSUM || ins.op == PO_RMAX)) ++reg_writes;
    }
    if (ins.op == PO_DIV || ins.op == PO_EXP || ins.op == PO_RSQRT) trans += (ins.flags & PF_SCALAR) ? 0 : 1;
    if (ins.op == PO_TANH || ins.op == PO_GELU || ins.op == PO_GELU_GRAD) trans += (ins.flags & PF_SCALAR) ? 0 : 2;
    return true;
  }

  // store of output tensor t (already defined) right now
  bool emit_store(int t) {
    const Tensor& T = g.tensors[t];
    ProgInstr s{};
    if (!operand(t, &s.a_kind, &s.a)) return false;
    s.aux = (uint8_t)T.store_as;
    if (val[t].kind == V_RSCAL) {
      if (n_rout >= kProgMaxOperands) return false;
      s.op = PO_STORE_SCAL;
      s.flags = PF_SCALAR;
      s.dst = (uint8_t)n_rout;
      rout_slot[n_rout++] = T.output_slot;
    } else if (val[t].kind == V_FULL) {
      if (n_out >= kProgMaxOperands) return false;
      s.op = PO_STORE;
      s.dst = (uint8_t)n_out;
      out_slot[n_out++] = T.output_slot;
    } else {
      return false;   // a column-shaped output would be written by every row
    }
    return emit(s);
  }

  bool run() {
    // anchor = the largest tensor
    int anchor = -1;
    for (size_t t = 0; t < g.tensors.size(); ++t)
      if (anchor < 0 || g.tensors[t].numel() > g.tensors[anchor].numel()) anchor = (int)t;
    if (anchor < 0) return false;
    const Tensor& a = g.tensors[anchor];
    rank = a.rank;
    for (int k = 0; k < rank; ++k) dims[k] = a.dims[k];
    cols = (uint32_t)dims[rank - 1];
    rows = (uint32_t)(a.numel() / cols);
    if (cols < 2) return false;

    // classes of all tensors; inputs by class
    int in_dt = -1;
    for (size_t t = 0; t < g.tensors.size(); ++t) {
      const Tensor& T = g.tensors[t];
      if (T.dtype == FS_I32) return false;
      val[t].kind = classify(T);
      val[t].root = (int)t;
      if (val[t].kind == V_NONE) return false;
    }
    for (int t : g.inputs) {
      const Tensor& T = g.tensors[t];
      if (val[t].kind == V_RSCAL) {
        if (rscal_in.size() >= kProgMaxOperands) return false;
        rscal_in.push_back(t);
      } else {
        if (in_dt >= 0 && T.dtype != in_dt) return false;   // one storage dtype for all vector inputs
        in_dt = T.dtype;
        std::vector<int32_t>& cls = val[t].kind == V_FULL ? full_in : col_in;
        if (cls.size() >= kProgMaxOperands) return false;
        cls.push_back(t);
      }
      if (T.output_slot >= 0) return false;   // an input handed straight to an output is no computation
    }
    p.dt = in_dt >= 0 ? in_dt : FS_F32;
    const uint32_t vec = 16u / (uint32_t)dtype_bytes(p.dt);
    if (cols % vec != 0) return false;
    p.rows = rows;
    p.cols = cols;

    // aliases and result classes; which ops read which roots
    const size_t n_ops = g.ops.size();
    std::vector<std::vector<int>> reads(n_ops);
    std::vector<char> emits_vec(n_ops, 0), emits_scal(n_ops, 0), is_alias(n_ops, 0);
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
          want = ka;
          break;
        case FS_BROADCAST:
          want = val[op.out].kind;   // whatever the stretched extents are, the storage is the source's
          is_alias[i] = 1;
          break;
        case FS_REDUCE_SUM: case FS_REDUCE_MAX: case FS_REDUCE_MEAN: {
          const Tensor& src = g.tensors[op.in[0]];
          if (op.axis != src.rank - 1) return false;              // only the row axis stays on chip
          if (ka == V_RSCAL) { want = V_RSCAL; is_alias[i] = 1; }  // reducing one element
          else if (ka == V_FULL) want = V_RSCAL;
          else return false;
          break;
        }
        default:
          return false;   // transposes move data between rows
      }
      if (is_alias[i]) {
        if (op.opcode == FS_BROADCAST) {
          // stretching may only go toward the pattern's row space
          if (val[op.out].kind != V_FULL && val[op.out].kind != ka) return false;
          val[op.out].kind = ka;          // keeps the source's class: readers broadcast it on the fly
        }
        val[op.out].root = val[op.in[0]].root;
      } else {
        if (val[op.out].kind != want) return false;
        reads[i].push_back(val[op.in[0]].root);
        if (op.n_in > 1) reads[i].push_back(val[op.in[1]].root);
        if (want == V_RSCAL) emits_scal[i] = 1;
        else emits_vec[i] = 1;
      }
      if (is_alias[i] && out.output_slot >= 0) reads[i].push_back(val[op.out].root);   // its store reads the root
    }
    // a broadcast result that is a graph output must be stored with full extents
    for (int t : g.outputs) {
      const Tensor& T = g.tensors[t];
      if (T.producer < 0) return false;
      if (g.ops[T.producer].opcode == FS_BROADCAST) {
        if (classify(T) != V_FULL) return false;
      }
    }

    for (size_t i = 0; i < n_ops; ++i)
      for (int r : reads[i]) val[r].last_read = (int)i;
    // look-ahead: a result needs a register if a reader comes after its accumulator was overwritten
    for (size_t i = 0; i < n_ops; ++i) {
      if (is_alias[i]) continue;
      const int r = g.ops[i].out;
      const bool scalar = is_scalar_shaped(val[r].kind);
      bool held = true;
      for (size_t j = i + 1; j < n_ops && !val[r].keep; ++j) {
        if (std::find(reads[j].begin(), reads[j].end(), r) != reads[j].end() && !held) val[r].keep = true;
        if (scalar ? emits_scal[j] : emits_vec[j]) held = false;
      }
    }

    // park the inputs
    p.n_full = (int32_t)full_in.size();
    p.n_col = (int32_t)col_in.size();
    p.n_rscal = (int32_t)rscal_in.size();
    for (size_t i = 0; i < full_in.size(); ++i) p.full_reg[i] = (uint8_t)(val[full_in[i]].reg = alloc(false));
    for (size_t i = 0; i < col_in.size(); ++i) val[col_in[i]].input_index = (int)i;
    for (size_t i = 0; i < rscal_in.size(); ++i) {
      p.rscal_sreg[i] = (uint8_t)(val[rscal_in[i]].reg = alloc(true));
      p.rscal_dt[i] = (uint8_t)g.tensors[rscal_in[i]].dtype;
    }
    for (int t : g.inputs)
      if (val[t].last_read < 0) release(t);   // declared but unread

    // emit
    for (size_t i = 0; i < n_ops; ++i) {
      const Op& op = g.ops[i];
      const Tensor& out = g.tensors[op.out];
      if (is_alias[i]) {
        if (out.output_slot >= 0) {
          // stored with the full extents of the output: a per-row or per-column source is stretched by the store
          const int saved = val[op.out].kind;
          if (op.opcode == FS_BROADCAST) val[op.out].kind = V_FULL;
          const bool ok = emit_store(op.out);
          val[op.out].kind = saved;
          if (!ok) return false;
        }
      } else {
        ProgInstr ins{};
        ins.b_kind = PK_IMM;
        if (!operand(op.in[0], &ins.a_kind, &ins.a)) return false;
        if (op.n_in > 1 && !operand(op.in[1], &ins.b_kind, &ins.b)) return false;
        const bool scalar = is_scalar_shaped(val[op.out].kind);
        if (scalar) ins.flags |= PF_SCALAR;
        bool mean = false;
        switch (op.opcode) {
          case FS_ADD: ins.op = PO_ADD; break;
          case FS_SUB: ins.op = PO_SUB; break;
          case FS_MUL: ins.op = PO_MUL; break;
          case FS_DIV: ins.op = PO_DIV; break;
          case FS_MAX: ins.op = PO_MAX; break;
          case FS_SCALE: ins.op = PO_MUL; ins.imm = (float)op.scalar; break;
          case FS_ADD_SCALAR: ins.op = PO_ADD; ins.imm = (float)op.scalar; break;
          case FS_SQUARE: ins.op = PO_SQUARE; break;
          case FS_EXP: ins.op = PO_EXP; break;
          case FS_RSQRT: ins.op = PO_RSQRT; break;
          case FS_TANH: ins.op = PO_TANH; break;
          case FS_GELU_TANH: ins.op = PO_GELU; break;
          case FS_GELU_TANH_GRAD: ins.op = PO_GELU_GRAD; break;
          case FS_CONVERT: ins.op = PO_CVT; ins.aux = (uint8_t)op.to_dtype; break;
          case FS_REDUCE_SUM: ins.op = PO_RSUM; break;
          case FS_REDUCE_MAX: ins.op = PO_RMAX; break;
          case FS_REDUCE_MEAN: ins.op = PO_RSUM; mean = true; break;
          default: return false;
        }
        // operands read for the last time give their registers back before the result takes one
        for (int r : reads[i])
          if (val[r].last_read == (int)i) release(r);
        Val& res = val[op.out];
        if (res.keep && !mean) {
          res.reg = alloc(scalar);
          ins.flags |= PF_KEEP;
          ins.dst = (uint8_t)res.reg;
        }
        if (!emit(ins)) return false;
        if (mean) {
          ProgInstr m{};
          m.op = PO_MUL;
          m.flags = PF_SCALAR;
          m.a_kind = PK_SACC;
          m.b_kind = PK_IMM;
          m.imm = (float)(1.0 / (double)cols);
          if (res.keep) {
            res.reg = alloc(true);
            m.flags |= PF_KEEP;
            m.dst = (uint8_t)res.reg;
          }
          if (!emit(m)) return false;
        }
        if (scalar) sacc_holds = op.out;
        else acc_holds = op.out;
        if (out.output_slot >= 0 && !emit_store(op.out)) return false;
      }
      if (is_alias[i])
        for (int r : reads[i])
          if (val[r].last_read == (int)i) release(r);
      if (p.n_regs > 250 || p.n_sregs > 250) return false;
    }
    return n_out + n_rout == (int)g.outputs.size();
  }
};

}  // namespace

bool build_row_program(const fs_graph& g, std::vector<Candidate>* out) {
  Compiler c(g);
  if (!c.run()) return false;
  const RowProgP& base = c.p;
  const int vec = 16 / dtype_bytes(base.dt);
  const uint32_t nvec = base.cols / vec;
  const double n = (double)base.rows * base.cols;
  const int64_t bytes_min = graph_bytes_min(g);

  struct Shape { uint32_t L; int K; bool block; };
  std::vector<Shape> shapes;
  for (int K : {1, 2, 4}) {
    uint32_t L = 1;
    while (L * (uint32_t)K < nvec) L <<= 1;
    if (L <= 64 && !(K > 1 && (uint64_t)L * K >= 2ull * nvec)) shapes.push_back({L, K, false});
  }
  if (c.n_reductions <= kProgMaxReductions)
    for (int K : {1, 2, 4})
      if (256ull * K >= nvec && 64ull * K < nvec) shapes.push_back({256, K, true});   // rows a wavefront cannot hold at this K

  for (const Shape& s : shapes) {
    const int kv = s.K * vec;
    const int64_t lds = (int64_t)base.n_regs * kv * 4 * 256 + (int64_t)base.n_col * base.cols * 4 +
                        (int64_t)base.n_sregs * 1024 + kProgMaxReductions * 16;
    if (lds > kProgMaxLdsBytes) continue;
    Candidate cand;
    memset(&cand.info, 0, sizeof cand.info);
    cand.info.scheme = s.block ? FS_SCHEME_LDS : (s.L == 1 ? FS_SCHEME_LOCAL : FS_SCHEME_WAVE);
    cand.info.n_kernels = 1;
    cand.info.bytes_min = bytes_min;
    cand.info.bytes_moved_model = bytes_min;
    snprintf(cand.info.pattern, sizeof cand.info.pattern, "row_program");
    cand.launches.emplace_back();
    Launch& l = cand.launches.back();
    l.kernel = K_ROW_PROGRAM;
    RowProgP q = base;
    q.lanes_per_row = (int32_t)s.L;
    int lg = 0;
    while ((1u << lg) < s.L) ++lg;
    q.lanes_log2 = lg;
    q.vecs_per_lane = s.K;
    l.args.u.prog = q;
    auto in_ref = [&](int32_t t) { BufRef r; r.kind = BUF_INPUT; r.slot = g.tensors[t].input_slot; return r; };
    for (size_t i = 0; i < c.full_in.size(); ++i) l.ptr[i] = in_ref(c.full_in[i]);
    for (size_t i = 0; i < c.col_in.size(); ++i) l.ptr[4 + i] = in_ref(c.col_in[i]);
    for (size_t i = 0; i < c.rscal_in.size(); ++i) l.ptr[8 + i] = in_ref(c.rscal_in[i]);
    for (int i = 0; i < c.n_out; ++i) { l.ptr[12 + i].kind = BUF_OUTPUT; l.ptr[12 + i].slot = c.out_slot[i]; }
    for (int i = 0; i < c.n_rout; ++i) { l.ptr[16 + i].kind = BUF_OUTPUT; l.ptr[16 + i].slot = c.rout_slot[i]; }
    const uint32_t rows_per_block = s.block ? 1 : 256 / s.L;
    l.shape.block[0] = 256;
    l.shape.grid[0] = (base.rows + rows_per_block - 1) / rows_per_block;
    l.shape.lds_bytes = (uint32_t)lds;
    cand.info.lanes_per_row = (int32_t)s.L;
    cand.info.vecs_per_lane = s.K;
    cand.info.rows_per_block = (int32_t)rows_per_block;
    cand.info.lds_bytes = (int32_t)lds;
    for (int k = 0; k < 3; ++k) { cand.info.block[k] = (int32_t)l.shape.block[k]; cand.info.grid[k] = (int32_t)l.shape.grid[k]; }
    snprintf(cand.info.kernel, sizeof cand.info.kernel, "row_program<%s,K%d,L%u,I%d,R%d>", dtype_name(base.dt), s.K, s.L,
             base.n_instr, base.n_regs);

    KernelCost kc;
    kc.hbm_bytes = (double)bytes_min;
    kc.cache_bytes = (double)c.col_in.size() * n * dtype_bytes(base.dt);
    kc.elems = n;
    // per element: the op itself plus operand / result moves; per instruction and wave: ~40 scalar-side cycles of dispatch
    const double dispatch = 40.0 * base.n_instr / (64.0 * kv) / 4.0;
    kc.valu_per_elem = 2.5 * c.vec_instr + dispatch + 2.0 * base.n_full;
    kc.trans_per_elem = c.trans;
    kc.lds_traffic_bytes = n * 4.0 * (c.reg_reads + c.reg_writes + base.n_full);
    kc.waves = (double)l.shape.grid[0] * 4;
    kc.waves_per_block = 4;
    kc.bytes_in_flight_per_lane = 16.0 * s.K * std::max(1, base.n_full);
    kc.vgpr_estimate = 40 + 3 * kv + 4 * s.K * (base.n_full <= 1 ? 1 : (base.n_full <= 2 ? 2 : 4));
    int steps = 0;
    for (uint32_t t = 1; t < std::min<uint32_t>(s.L, 64); t <<= 1) ++steps;
    kc.xlane_steps = steps * c.n_reductions;
    kc.barriers = s.block ? c.n_reductions : 0;
    kc.lds_bytes_per_block = (int32_t)lds;
    kc.lane_utilisation = (double)nvec / ((double)s.L * s.K);
    kc.access_run_bytes = s.L >= 8 ? 0 : s.L * 16.0;
    kc.preamble_instr = 60;
    cand.cost = kc;
    out->push_back(cand);
  }
  return !out->empty();
}

}  // namespace fs
