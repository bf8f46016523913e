// Code generator for row patterns (paper Section 4: "the code generator takes a fusion
// pattern as input and produces a GPU kernel").  Input is the instruction list the row-program
// compiler made for the pattern (an accumulator machine over full-shaped and per-row values);
// output is HIP source of ONE straight-line kernel specialised to the pattern, its extents
// and its launch shape: every kept value is a named array of registers, so the device
// compiler does the register allocation and scheduling that the interpreter pays for at
// run time with an LDS register file and a dispatch per instruction.  The source is
// compiled at plan time by the run-time compiler (kernels/gen_runtime.hip).
#include <algorithm>
#include <cstring>
#include <string>
#include <vector>

#include "fs_internal.hpp"

namespace fs {
namespace {

#include "build/embedded_sources.inc"   // kEmbeddedDeviceUtils, kEmbeddedGenSupport: the two device headers as text

const char* storage_type(int dt) {
  switch (dt) {
    case DT_F16: return "f16_t";
    case DT_BF16: return "bf16_t";
    default: return "float";
  }
}

// a float as source text that compiles back to the same bits
std::string literal(float v) {
  uint32_t u;
  memcpy(&u, &v, 4);
  char b[96];
  snprintf(b, sizeof b, "__builtin_bit_cast(float, 0x%08xu /* %.9g */)", u, (double)v);
  return b;
}

std::string fmt(const char* f, ...) __attribute__((format(printf, 1, 2)));
std::string fmt(const char* f, ...) {
  char b[512];
  va_list ap;
  va_start(ap, f);
  vsnprintf(b, sizeof b, f, ap);
  va_end(ap);
  return b;
}

// `a` (op) `b` as an expression; a is the accumulator's element, b the other operand
std::string expression(int op, const std::string& a, const std::string& b, int aux) {
  switch (op) {
    case PO_ADD: return a + " + " + b;
    case PO_SUB: return a + " - " + b;
    case PO_RSUB: return b + " - " + a;
    case PO_MUL: return a + " * " + b;
    case PO_DIV: return a + " * fast_rcp(" + b + ")";
    case PO_RDIV: return b + " * fast_rcp(" + a + ")";
    case PO_MAX: return "fmaxf(" + a + ", " + b + ")";
    case PO_SQUARE: return a + " * " + a;
    case PO_EXP: return "fast_exp(" + a + ")";
    case PO_RSQRT: return "fast_rsqrt(" + a + ")";
    case PO_TANH: return "fast_tanh(" + a + ")";
    case PO_GELU: return "gelu_fwd(" + a + ")";
    case PO_GELU_GRAD: return "gelu_grad(" + a + ")";
    case PO_LOG: return "full_log(" + a + ")";
    case PO_SIGMOID: return "fast_sigmoid(" + a + ")";
    case PO_RELU: return "fmaxf(" + a + ", 0.0f)";
    case PO_ABS: return "__builtin_fabsf(" + a + ")";
    case PO_SQRT: return "full_sqrt(" + a + ")";
    case PO_CVT: return fmt("gen_round<%d>(", aux) + a + ")";
    default: return b;   // PO_LOAD
  }
}

// row index of an operand stretched or permuted along the leading axes, from the row's index (lead0, lead1, lead2) along them
std::string stretched_row(const uint32_t (&ms)[3], const char* pre = "") {
  return fmt("(size_t)(%slead0 * %uu + %slead1 * %uu + %slead2 * %uu)", pre, ms[0], pre, ms[1], pre, ms[2]);
}

}  // namespace

// online[q] = 1 where reductions q and q + 1 of the program are "rmax; acc - max; exp; rsum" (a chunked row gathers both
// in one pass); returns the number of such pairs.  `online` may be null.
int online_reduction_pairs(const RowProgP& p, std::vector<char>* online) {
  int q = 0, pairs = 0;
  bool previous = false;
  for (int i = 0; i < p.n_instr; ++i) {
    const ProgInstr& in = p.instr[i];
    if (in.op != PO_RSUM && in.op != PO_RMAX && in.op != PO_RSUMSQ) continue;
    const bool pair = in.op == PO_RMAX && i + 3 < p.n_instr && p.instr[i + 1].op == PO_SUB && p.instr[i + 1].b_kind == PK_SACC &&
                      !(p.instr[i + 1].flags & PF_SCALAR) && p.instr[i + 2].op == PO_EXP && !(p.instr[i + 2].flags & PF_SCALAR) &&
                      p.instr[i + 3].op == PO_RSUM && !previous;
    if (pair) {
      ++pairs;
      if (online && q < (int)online->size()) (*online)[q] = 1;
    }
    previous = pair;
    ++q;
  }
  return pairs;
}

namespace {
// member = false: an extern "C" kernel `entry(const GenArgs a)`.  member = true: a device function
// `entry(const GenArgs& a, uint32_t fs_block)` that a packed kernel calls for the member's range of workgroups.
std::string body_with_entry(const RowProgP& p, const char* entry, bool member = false);
const char kEntryPlaceholder[] = "@ENTRY@";
uint32_t fnv1a(const std::string& text) {
  uint32_t h = 2166136261u;
  for (unsigned char ch : text) h = (h ^ ch) * 16777619u;
  return h;
}
}  // namespace

// The kernel's name carries a hash of its own source (pattern, extents and launch shape), so that kernel traces
// tell the generated kernels of a process apart.
std::string generated_kernel_entry(const RowProgP& p) {
  return fmt("fs_gen_row_%08x", fnv1a(body_with_entry(p, kEntryPlaceholder)));
}

std::string generate_row_kernel_body(const RowProgP& p) { return body_with_entry(p, generated_kernel_entry(p).c_str()); }

namespace {
// Source text of one instruction of the accumulator machine (see ProgInstr): an unrolled loop over the lane's elements
// for full-shaped work, a scalar statement for per-row work, a call into GenRow for reductions and stores.
// A pass over a row that is worked through in chunks (see chunked_body): reductions before `reduction` are known
// (red<q>), that one gathers the lanes' partial values and ends the pass; stores happen in the last pass only.
struct ChunkPass {
  int reduction;      // the reduction this pass is for; the number of reductions = the last pass, with the stores
  bool last_pass, last_chunk;
  bool ended = false; // set when the pass's reduction has been emitted: nothing after it belongs to the pass
  bool online = false;   // the pass's reduction is a row maximum whose only use is exp(acc - max) summed over the row: one
                         // pass gathers both, the sum under a running maximum (see chunked_body)
};

// Ends a chunk's share of a pass: the running values pass through an empty asm statement.  Such statements keep their
// order, and each chunk's kept registers pass through one before they are unpacked, so no chunk's unpacking starts
// before the chunk before it is folded into the running values.  Without it the compiler unpacks several chunks ahead
// to hide latency, and a row kept in registers no longer fits (it spills by hundreds of bytes per lane).
std::string kChunkOrderPin(const char* a, const char* b) {
  return b ? fmt("  asm volatile(\"\" : \"+v\"(%s), \"+v\"(%s));\n", a, b) : fmt("  asm volatile(\"\" : \"+v\"(%s));\n", a);
}

std::string instruction_text(const RowProgP& p, const ProgInstr& in, bool block, int n_waves, int* reduction_no, ChunkPass* cp = nullptr) {
  std::string t;
  const bool scalar = (in.flags & PF_SCALAR) != 0, keep = (in.flags & PF_KEEP) != 0;
  if (cp) {
    if ((in.op == PO_STORE && !cp->last_pass) || (in.op == PO_STORE_SCAL && !(cp->last_pass && cp->last_chunk))) return t;
    if (in.op == PO_RSUM || in.op == PO_RMAX || in.op == PO_RSUMSQ) {
      const int q = (*reduction_no)++;
      if (q < cp->reduction) {
        t += fmt("  sacc = red%d;\n", q);
        if (keep) t += fmt("  s%d = sacc;\n", in.dst);
      } else if (cp->online) {
        // the lane's running maximum m_run and the lane's sum s_run of exp(acc - m_run) over the chunks seen so far: a
        // new chunk first raises the maximum (the sum so far is rescaled by exp(old - new), one exponential per lane and
        // chunk), then adds its own exponentials.  Padding lanes hold -huge for the maximum and add nothing to the sum;
        // the floor keeps the difference of two "nothing yet" maxima at zero instead of inf - inf.
        t += "  {\n  const float m_new = fmaxf(m_run, fmaxf(row.partial<OpMax, true, false>(acc), -3.4028234664e38f));\n";
        t += "#pragma unroll\n  for (int j = 0; j < KV; ++j) acc[j] = fast_exp(acc[j] - m_new);\n";
        t += "  s_run = s_run * fast_exp(m_run - m_new) + row.partial<OpSum, false, false>(acc);\n  m_run = m_new;\n  }\n";
        t += kChunkOrderPin("m_run", "s_run");
        ++*reduction_no;   // the sum's turn is taken as well
        cp->ended = true;
      } else {
        const bool is_max = in.op == PO_RMAX;
        t += fmt("  part = %s::apply(part, row.partial<%s, %s, %s>(acc));\n", is_max ? "OpMax" : "OpSum", is_max ? "OpMax" : "OpSum",
                 is_max ? "true" : "false", in.op == PO_RSUMSQ ? "true" : "false");
        t += kChunkOrderPin("part", nullptr);
        cp->ended = true;
      }
      return t;
    }
  }
  switch (in.op) {
    case PO_STORE:
      if ((p.out_perm >> in.dst) & 1u)   // stored through a folded transpose: the row lands at its permuted place
        t += fmt("  row.store_at<%s>(a.out[%d], %s, acc);\n", storage_type(in.aux), in.dst, stretched_row(p.oms[in.dst]).c_str());
      else
        t += fmt("  row.store<%s>(a.out[%d], acc);\n", storage_type(in.aux), in.dst);
      return t;
    case PO_STORE_SCAL:
      t += fmt("  row.store_scalar<%s>(a.rout[%d], sacc);\n", storage_type(in.aux), in.dst);
      return t;
    case PO_COLSUM:
      t += fmt("  row.colsum_add(acc, cs%d);\n", in.dst);
      return t;
    case PO_RSUM: case PO_RMAX: case PO_RSUMSQ: {
      const bool is_max = in.op == PO_RMAX;
      const std::string slot = block ? fmt("slots + %d", n_waves * *reduction_no) : std::string("nullptr");
      t += fmt("  sacc = row.reduce<%s, %s, %s>(acc, %s);\n", is_max ? "OpMax" : "OpSum", is_max ? "true" : "false",
               in.op == PO_RSUMSQ ? "true" : "false", slot.c_str());
      ++*reduction_no;
      if (keep) t += fmt("  s%d = sacc;\n", in.dst);
      return t;
    }
    default:
      break;
  }
  if (scalar) {
    const std::string b = in.b_kind == PK_SCAL ? fmt("s%d", in.b) : (in.b_kind == PK_SACC ? std::string("sacc") : literal(in.imm));
    t += "  sacc = " + expression(in.op, "sacc", b, in.aux) + ";\n";
    if (keep) t += fmt("  s%d = sacc;\n", in.dst);
    return t;
  }
  std::string b;
  switch (in.b_kind) {
    case PK_REG: b = fmt("r%d[j]", in.b); break;
    case PK_COL: b = fmt("c%d[j]", in.b); break;
    case PK_ACC: b = "acc[j]"; break;
    case PK_SCAL: b = fmt("s%d", in.b); break;
    case PK_SACC: b = "sacc"; break;
    default: b = literal(in.imm); break;
  }
  t += "#pragma unroll\n  for (int j = 0; j < KV; ++j) acc[j] = " + expression(in.op, "acc[j]", b, in.aux) + ";\n";
  if (keep) t += fmt("#pragma unroll\n  for (int j = 0; j < KV; ++j) r%d[j] = acc[j];\n", in.dst);
  return t;
}

// A row longer than the lanes' registers hold (beyond 1024 threads x 8 steps) is worked through in chunks of
// lanes x steps elements, one pass over the row per row reduction and a last one for the stores.  Every pass runs
// the instruction list from the start up to its reduction on each chunk, with the reductions of earlier passes
// replaced by their results; what a pass does not need of that (other operands' loads, values kept for later
// stores) is dead code to the device compiler.  The operands are read once per pass: the re-reads are the price of
// keeping the pattern in one kernel (Section 4.2 keeps such a value on chip; a row of this length has no chip
// memory to stay in), and they come from the caches as far as the rows in flight fit there.
std::string chunked_body(const RowProgP& p, const char* entry) {
  const uint32_t L = (uint32_t)p.lanes_per_row, chunk = L * (uint32_t)p.vecs_per_lane * (uint32_t)p.vec, NC = (uint32_t)p.col_chunks;
  const uint32_t tail = p.cols - (NC - 1u) * chunk;
  const int n_waves = (int)(L / 64u);
  std::vector<int> is_max;
  for (int i = 0; i < p.n_instr; ++i)
    if (p.instr[i].op == PO_RSUM || p.instr[i].op == PO_RMAX || p.instr[i].op == PO_RSUMSQ) is_max.push_back(p.instr[i].op == PO_RMAX);
  const int n_red = (int)is_max.size();
  // A row maximum that is only there to keep the exponentials in range -- rmax; acc - max; exp; rsum, the core of every
  // softmax -- does not need a pass of its own: sum_j exp(x_j - M) = sum over chunks of exp(m - M) * sum_j exp(x_j - m)
  // for any m, so one pass gathers the maximum and the sum together (a running maximum per lane, the sum rescaled when
  // it rises), and the pattern takes one pass over the row less.  online[q]: reductions q and q + 1 are such a pair.
  std::vector<char> online(n_red + 1, 0);
  online_reduction_pairs(p, &online);
  std::string s = "using namespace fsk;\n";
  s += fmt("extern \"C\" __global__ void __launch_bounds__(%u) %s(const GenArgs a) {\n", L, entry);
  s += "  const uint32_t fs_block = blockIdx.x;\n";
  s += fmt("  typedef GenRow<%uu, %uu, %d, %d, %uu, true, 1u, %uu> Row;       // a whole chunk\n", p.rows, chunk, p.vec, p.vecs_per_lane, L, p.cols);
  s += fmt("  typedef GenRow<%uu, %uu, %d, %d, %uu, true, 1u, %uu> TailRow;   // the row's last chunk\n", p.rows, tail, p.vec, p.vecs_per_lane, L, p.cols);
  s += "  constexpr int KV = Row::KV;\n";
  if (n_red > 0) s += fmt("  __shared__ float slots[%d];\n", n_waves * n_red);
  for (int q = 0; q < n_red; ++q) s += fmt("  float red%d;\n", q);
  s += "  const Row row0(fs_block);\n";
  if ((p.full_bcast | p.rscal_bcast | p.out_perm) != 0)
    s += fmt("  const uint32_t q1 = row0.row_c / %uu, lead2 = row0.row_c - q1 * %uu, lead0 = q1 / %uu, lead1 = q1 - lead0 * %uu;\n", p.od[2].d,
             p.od[2].d, p.od[1].d, p.od[1].d);
  for (int i = 0; i < p.n_rscal; ++i) {
    const std::string at = ((p.rscal_bcast >> i) & 1u) ? stretched_row(p.rms[i]) : std::string("(size_t)row0.row_c");
    s += fmt("  const float in_rscal%d = load1(static_cast<const %s*>(a.rscal[%d]) + %s);\n", i, storage_type(p.rscal_dt[i]), i, at.c_str());
  }
  // The first `kept` chunks stay in registers, in storage form, from the first pass on: 1024 lanes hold more of a
  // row in their registers (64 of them hold 256 KB) than the compute unit's LDS would, and later passes then read
  // nothing of those chunks again.  Register arrays cannot be indexed at run time, so the kept chunks are written
  // out one by one; the others are walked by a loop.
  const uint32_t kept = (uint32_t)std::max(0, std::min(p.col_kept, p.col_chunks));
  for (uint32_t c = 0; c < kept; ++c)
    for (int i = 0; i < p.n_full; ++i)
      s += fmt("  %s::Raw<%s> kept%d_%u;\n", c == NC - 1u ? "TailRow" : "Row", storage_type(p.full_dt[i]), i, c);
  // one chunk's share of a pass, for the row object `row` in scope; kept_chunk >= 0: that chunk stays in registers
  auto piece = [&](int pass, bool last_chunk, int kept_chunk, bool preloaded = false) {
    std::string t;
    const bool last_pass = pass == n_red;
    for (int i = 0; i < p.n_full; ++i) {
      const bool stretched = ((p.full_bcast >> i) & 1u) != 0;
      const std::string at = stretched ? stretched_row(p.ms[i]) : std::string("(size_t)row.row_c");
      if (kept_chunk >= 0 && (pass > 0 || preloaded)) {
        // (the compiler must not carry the unpacked form over from the pass before: that would take the registers twice)
        t += fmt("  kept%d_%d.forget_contents();\n  const auto& raw_full%d = kept%d_%d;\n", i, kept_chunk, i, i, kept_chunk);
        continue;
      }
      // an operand is read for the last time in the last pass, or in the first one where its chunk is kept
      const bool once = !stretched && (last_pass || kept_chunk >= 0);
      t += fmt("  const auto raw_full%d = row.load<%s, %s>(a.full[%d], %s);\n", i, storage_type(p.full_dt[i]), once ? "true" : "false", i,
               at.c_str());
      if (kept_chunk >= 0) t += fmt("  kept%d_%d = raw_full%d;\n", i, kept_chunk, i);
    }
    for (int i = 0; i < p.n_col; ++i)
      t += fmt("  const auto raw_col%d = row.load<%s, false>(a.col[%d], 0);\n", i, storage_type(p.col_dt[i]), i);
    t += "  float acc[KV], sacc = 0.0f;\n#pragma unroll\n  for (int j = 0; j < KV; ++j) acc[j] = 0.0f;\n";
    for (int r = 0; r < p.n_regs; ++r) t += fmt("  float r%d[KV];\n", r);
    for (int r = 0; r < p.n_sregs; ++r) t += fmt("  float s%d = 0.0f;\n", r);
    for (int i = 0; i < p.n_col; ++i) t += fmt("  float c%d[KV];\n  row.unpack_to<%s>(raw_col%d, c%d);\n", i, storage_type(p.col_dt[i]), i, i);
    for (int i = 0; i < p.n_full; ++i) {
      const bool parked = p.full_reg[i] != 255, to_acc = p.acc_input == i;
      if (parked) {
        t += fmt("  row.unpack_to<%s>(raw_full%d, r%d);\n", storage_type(p.full_dt[i]), i, p.full_reg[i]);
        if (to_acc) t += fmt("#pragma unroll\n  for (int j = 0; j < KV; ++j) acc[j] = r%d[j];\n", p.full_reg[i]);
      } else if (to_acc) {
        t += fmt("  row.unpack_to<%s>(raw_full%d, acc);\n", storage_type(p.full_dt[i]), i);
      }
    }
    for (int i = 0; i < p.n_rscal; ++i) t += fmt("  s%d = in_rscal%d;\n", p.rscal_sreg[i], i);
    ChunkPass cp{pass, last_pass, last_chunk};
    cp.online = !last_pass && online[pass] != 0;
    int reduction_no = 0;
    for (int i = 0; i < p.n_instr && !cp.ended; ++i) t += instruction_text(p, p.instr[i], true, n_waves, &reduction_no, &cp);
    return t;
  };
  int walk = 0;   // passes emitted so far (a fused pair counts once): every other one walks the row backwards
  for (int pass = 0; pass <= n_red; ++pass, ++walk) {
    const bool fused = pass < n_red && online[pass] != 0;
    s += "  {\n";
    if (fused) s += "  float m_run = -3.4028234664e38f, s_run = 0.0f;\n";
    else if (pass < n_red) s += fmt("  float part = %s;\n", is_max[pass] ? "-__builtin_huge_valf()" : "0.0f");
    // the kept chunks, one block each
    std::string in_registers;
    // A first pass that also exponentiates (a fused maximum + sum) has more live values per chunk than one that only
    // compares; left to itself the compiler interleaves the chunks' arithmetic and runs out of registers.  So the loads
    // of all kept chunks are issued first, and the chunks are then worked through one after the other, each behind a
    // scheduling barrier (a chunk's arithmetic starts when its own loads have landed).
    const bool preload = fused && pass == 0 && kept > 0;
    if (preload) {
      for (uint32_t c = 0; c < kept; ++c)
        for (int i = 0; i < p.n_full; ++i) {
          const bool stretched = ((p.full_bcast >> i) & 1u) != 0;
          const std::string at = stretched ? stretched_row(p.ms[i]) : std::string("(size_t)row.row_c");
          in_registers += fmt("  {\n  const %s row(fs_block, 0, %uu);\n  kept%d_%u = row.load<%s, %s>(a.full[%d], %s);\n  }\n", c == NC - 1u ? "TailRow" : "Row",
                              c * chunk, i, c, storage_type(p.full_dt[i]), stretched ? "false" : "true", i, at.c_str());
        }
      in_registers += "  __builtin_amdgcn_sched_barrier(0);\n";
    }
    for (uint32_t c = 0; c < kept; ++c) {
      const bool is_tail = c == NC - 1u;
      in_registers += fmt("  {\n  const %s row(fs_block, 0, %uu);\n", is_tail ? "TailRow" : "Row", c * chunk) + piece(pass, is_tail, (int)c, preload) + "  }\n";
      if (preload) in_registers += "  __builtin_amdgcn_sched_barrier(0);\n";
    }
    // the others: whole chunks by a loop, then the row's last chunk.  Every other pass walks them backwards: it
    // starts with the chunks the pass before read last, which the caches are likeliest to hold still
    const bool backwards = (walk & 1) != 0;
    std::string from_memory_whole, from_memory_last;
    if (kept < NC - 1u)
      from_memory_whole = fmt("#pragma unroll 1\n  for (uint32_t chunk = %uu; chunk < %uu; ++chunk) {\n  const Row row(fs_block, 0, %s * %uu);\n",
                              kept, NC - 1u, backwards ? fmt("(%uu - chunk)", NC - 2u + kept).c_str() : "chunk", chunk) +
                          piece(pass, false, -1) + "  }\n";
    if (kept < NC) from_memory_last = fmt("  {\n  const TailRow row(fs_block, 0, %uu);\n", (NC - 1u) * chunk) + piece(pass, true, -1) + "  }\n";
    s += backwards ? from_memory_last + from_memory_whole + in_registers : in_registers + from_memory_whole + from_memory_last;
    if (fused) {
      // the lanes' maxima meet first; every lane then brings its sum to the row's maximum before the sums meet
      s += fmt("  red%d = Row::finish<OpMax>(m_run, slots + %d);\n", pass, n_waves * pass);
      s += fmt("  red%d = Row::finish<OpSum>(s_run * fast_exp(m_run - red%d), slots + %d);\n", pass + 1, pass, n_waves * (pass + 1));
      ++pass;   // the sum's pass is done as well
    } else if (pass < n_red) {
      s += fmt("  red%d = Row::finish<%s>(part, slots + %d);\n", pass, is_max[pass] ? "OpMax" : "OpSum", n_waves * pass);
    }
    s += "  }\n";
  }
  s += "}\n";
  return s;
}

std::string body_with_entry(const RowProgP& p, const char* entry, bool member) {
  if (p.col_chunks > 1) return chunked_body(p, entry);   // never a pack member: more than 256 threads
  const bool block = p.lanes_per_row > 64;
  int n_reductions = 0;
  for (int i = 0; i < p.n_instr; ++i)
    if (p.instr[i].op == PO_RSUM || p.instr[i].op == PO_RMAX || p.instr[i].op == PO_RSUMSQ) ++n_reductions;

  std::string s;
  if (member) {
    s += fmt("static __device__ __forceinline__ void %s(const GenArgs& a, const uint32_t fs_block) {\n", entry);
  } else {
    s += "using namespace fsk;\n";
    s += fmt("extern \"C\" __global__ void __launch_bounds__(%d) %s(const GenArgs a) {\n", block ? p.lanes_per_row : 256, entry);
    s += "  const uint32_t fs_block = blockIdx.x;\n";
  }
  const uint32_t R = p.rows_per_group > 1 ? (uint32_t)p.rows_per_group : 1u;
  const uint32_t CT = p.col_tiles > 1 ? (uint32_t)p.col_tiles : 1u;   // column tiles of cols / CT elements
  s += fmt("  typedef GenRow<%uu, %uu, %d, %d, %uu, %s, %uu, %uu> Row;\n", p.rows, p.cols / CT, p.vec, p.vecs_per_lane,
           (uint32_t)p.lanes_per_row, block ? "true" : "false", R, p.cols);
  s += "  constexpr int KV = Row::KV;\n";
  const int n_waves = block ? p.lanes_per_row / 64 : 4;
  const bool looped = p.n_colsum > 0;
  // a workgroup that walks several rows alternates between two sets of reduction slots: a wave may write the next
  // row's partial value while a slower one still reads this row's, and nobody can be two rows ahead (the next row's
  // own barrier stands in between), so no barrier is needed at a row's end
  if (block && n_reductions > 0)
    s += looped ? fmt("  __shared__ float slots_all[%d];\n", 2 * n_waves * n_reductions) : fmt("  __shared__ float slots[%d];\n", n_waves * n_reductions);
  const bool needs_lead = (p.full_bcast | p.rscal_bcast | p.out_perm) != 0;
  // the row's index along the leading axes, for the row object `rv`; names carry the prefix `pre`
  auto lead_of = [&](const char* rv, const char* pre, bool declare) {
    return fmt("  %s%sq1 = %s.row_c / %uu, %slead2 = %s.row_c - %sq1 * %uu, %slead0 = %sq1 / %uu, %slead1 = %sq1 - %slead0 * %uu;\n",
               declare ? "const uint32_t " : "", pre, rv, p.od[2].d, pre, rv, pre, p.od[2].d, pre, pre, p.od[1].d, pre, pre, pre, p.od[1].d);
  };
  // the loads of one row's operands (everything but the column vectors); `decl` declares the variables or is empty
  auto row_loads = [&](const char* rv, const char* pre, const char* decl_raw, const char* decl_scalar) {
    std::string t;
    for (int i = 0; i < p.n_full; ++i) {
      // an input stretched along leading axes is read by many rows: it goes through the caches like a column vector;
      // the others are read once and stream past them
      const bool stretched = ((p.full_bcast >> i) & 1u) != 0;
      const std::string at = stretched ? stretched_row(p.ms[i], pre) : fmt("(size_t)%s.row_c", rv);
      t += fmt("  %s%sraw_full%d = %s.load<%s, %s>(a.full[%d], %s);\n", decl_raw, pre, i, rv, storage_type(p.full_dt[i]),
               stretched ? "false" : "true", i, at.c_str());
    }
    for (int i = 0; i < p.n_rscal; ++i) {
      const std::string at = ((p.rscal_bcast >> i) & 1u) ? stretched_row(p.rms[i], pre) : fmt("(size_t)%s.row_c", rv);
      t += fmt("  %s%sin_rscal%d = load1(static_cast<const %s*>(a.rscal[%d]) + %s);\n", decl_scalar, pre, i, storage_type(p.rscal_dt[i]), i,
               at.c_str());
    }
    return t;
  };
  auto col_loads = [&](const char* rv) {
    std::string t;
    for (int i = 0; i < p.n_col; ++i)
      t += fmt("  const auto raw_col%d = %s.load<%s, false>(a.col[%d], 0);\n", i, rv, storage_type(p.col_dt[i]), i);
    return t;
  };
  auto col_unpack = [&](const char* rv) {
    std::string t;
    for (int i = 0; i < p.n_col; ++i) {
      t += fmt("  float c%d[KV];\n", i);
      t += fmt("  %s.unpack_to<%s>(raw_col%d, c%d);\n", rv, storage_type(p.col_dt[i]), i, i);
    }
    return t;
  };
  if (looped) {
    // Running column sums live across the rows a lane group works through; the rows' own work is one round.
    // The rounds are software-pipelined: the next row's loads are issued before this row's arithmetic starts, and the
    // column vectors are loaded once.  The first and the last round stand outside the loop.  The counter a wave waits
    // on counts loads and stores in issue order; at the head of a loop whose first entry comes from code that issued
    // loads last and whose back edge comes from a round that issued its store last, the compiler has to wait for
    // everything, the store included, in every round.  With the first round peeled both ways into the loop look
    // alike and the wait leaves the stores in flight; the last round has no row to load ahead.
    if (!block) s += fmt("  __shared__ float colred[%d][4 * Row::PADDED_COLS];\n", p.n_colsum);
    for (int i = 0; i < p.n_colsum; ++i)
      s += fmt("  float cs%d[KV];\n#pragma unroll\n  for (int j = 0; j < KV; ++j) cs%d[j] = 0.0f;\n", i, i);
    // neighbouring workgroups take neighbouring column tiles of the same rows
    if (CT > 1) s += fmt("  const uint32_t tile = blockIdx.x %% %uu, row_wg = blockIdx.x / %uu, n_row_wgs = gridDim.x / %uu;\n", CT, CT, CT);
    else s += "  const uint32_t tile = 0, row_wg = blockIdx.x, n_row_wgs = gridDim.x;\n";
    s += "  Row nrow(row_wg, tile);\n";
    s += col_loads("nrow");
    if (needs_lead) s += "  uint32_t nq1, nlead0, nlead1, nlead2;\n" + lead_of("nrow", "n", false);
    s += row_loads("nrow", "n", "auto ", "float ");
    s += col_unpack("nrow");
    s += "  auto round = [&](const uint32_t it, auto has_next) {\n";
    if (block && n_reductions > 0) s += fmt("  float* const slots = slots_all + (it & 1u) * %du;\n", n_waves * n_reductions);
    s += "  const Row row = nrow;\n";
    if (p.out_perm) s += lead_of("row", "", true);
    for (int i = 0; i < p.n_full; ++i) s += fmt("  const auto raw_full%d = nraw_full%d;\n", i, i);
    for (int i = 0; i < p.n_rscal; ++i) s += fmt("  const float in_rscal%d = nin_rscal%d;\n", i, i);
    s += "  if constexpr (decltype(has_next)::value) {\n";
    s += "  nrow = Row((it + 1u) * n_row_wgs + row_wg, tile);\n";
    if (needs_lead) s += lead_of("nrow", "n", false);
    s += row_loads("nrow", "n", "", "");
    s += "  }\n";
  } else {
    s += "  const Row row(fs_block);\n";
    // ---- every global load is issued before anything waits
    if (needs_lead) s += lead_of("row", "", true);
    s += row_loads("row", "", "const auto ", "const float ");
    s += col_loads("row");
  }

  // ---- values: the accumulators, the kept full-shaped values, the column vectors, the kept per-row values
  s += "  float acc[KV], sacc = 0.0f;\n";
  s += "#pragma unroll\n  for (int j = 0; j < KV; ++j) acc[j] = 0.0f;\n";
  for (int r = 0; r < p.n_regs; ++r) s += fmt("  float r%d[KV];\n", r);
  for (int r = 0; r < p.n_sregs; ++r) s += fmt("  float s%d = 0.0f;\n", r);
  if (!looped) s += col_unpack("row");
  for (int i = 0; i < p.n_full; ++i) {
    const bool parked = p.full_reg[i] != 255;
    const bool to_acc = p.acc_input == i;
    if (parked) {
      s += fmt("  row.unpack_to<%s>(raw_full%d, r%d);\n", storage_type(p.full_dt[i]), i, p.full_reg[i]);
      if (to_acc) s += fmt("#pragma unroll\n  for (int j = 0; j < KV; ++j) acc[j] = r%d[j];\n", p.full_reg[i]);
    } else if (to_acc) {
      s += fmt("  row.unpack_to<%s>(raw_full%d, acc);\n", storage_type(p.full_dt[i]), i);
    }
  }
  for (int i = 0; i < p.n_rscal; ++i) s += fmt("  s%d = in_rscal%d;\n", p.rscal_sreg[i], i);

  // ---- the pattern's ops, in the order of the instruction list
  int reduction_no = 0;
  for (int i = 0; i < p.n_instr; ++i) s += instruction_text(p, p.instr[i], block, n_waves, &reduction_no);
  if (looped) {
    s += "  };\n";
    if (R > 1u) s += "  round(0u, Yes{});\n";
    if (R > 2u) s += fmt("#pragma unroll 1\n  for (uint32_t it = 1u; it < %uu; ++it) round(it, Yes{});\n", R - 1u);
    s += fmt("  round(%uu, No{});\n", R - 1u);
    for (int i = 0; i < p.n_colsum; ++i)
      s += fmt("  Row::colsum_flush(cs%d, %s, static_cast<float*>(a.ws) + (size_t)row_wg * %uu + %uu + tile * %uu);\n", i,
               block ? "nullptr" : fmt("colred[%d]", i).c_str(), (uint32_t)p.n_colsum * p.cols, (uint32_t)i * p.cols, p.cols / CT);
  }
  s += "}\n";
  return s;
}
}  // namespace

// One kernel over several independent row patterns (kernel packing, Section 4.1, across patterns): every member is
// a device function made from its own row program; a workgroup finds its member from its index (the members own
// consecutive ranges of workgroups) and runs it with a virtual workgroup index.  The operand pointers of all members
// travel in one table in the kernel arguments; `ptr_slots[m]` lists, for member m, the row-program pointer slots
// (kSlot*) behind its consecutive table entries.
std::string generate_pack_kernel(const std::vector<RowProgP>& members, const std::vector<uint32_t>& blocks,
                                 std::vector<std::vector<int>>* ptr_slots, std::string* entry) {
  std::string body;
  ptr_slots->assign(members.size(), {});
  size_t n_ptrs = 0;
  for (size_t m = 0; m < members.size(); ++m) {
    const RowProgP& p = members[m];
    std::vector<int>& slots = (*ptr_slots)[m];
    for (int i = 0; i < p.n_full; ++i) slots.push_back(kSlotFull + i);
    for (int i = 0; i < p.n_col; ++i) slots.push_back(kSlotCol + i);
    for (int i = 0; i < p.n_rscal; ++i) slots.push_back(kSlotRscal + i);
    for (int i = 0; i < p.n_instr; ++i) {
      if (p.instr[i].op == PO_STORE) slots.push_back(kSlotOut + p.instr[i].dst);
      if (p.instr[i].op == PO_STORE_SCAL) slots.push_back(kSlotRout + p.instr[i].dst);
    }
    n_ptrs += slots.size();
    body += body_with_entry(p, fmt("fs_member_%zu", m).c_str(), true);
  }
  std::string k;
  k += fmt("struct PackPtrs { void* p[%zu]; };\n", std::max<size_t>(n_ptrs, 1));
  k += fmt("extern \"C\" __global__ void __launch_bounds__(256) %s(const PackPtrs t) {\n", kEntryPlaceholder);
  k += "  const uint32_t b = blockIdx.x;\n";
  size_t at = 0;
  uint32_t first = 0;
  for (size_t m = 0; m < members.size(); ++m) {
    k += fmt("  if (b < %uu) {\n    GenArgs a{};\n", first + blocks[m]);
    for (int slot : (*ptr_slots)[m]) {
      const char* field = slot >= kSlotRout ? "rout" : slot >= kSlotOut ? "out" : slot >= kSlotRscal ? "rscal" : slot >= kSlotCol ? "col" : "full";
      k += fmt("    a.%s[%d] = t.p[%zu];\n", field, slot % 8, at++);
    }
    k += fmt("    fs_member_%zu(a, b - %uu);\n    return;\n  }\n", m, first);
    first += blocks[m];
  }
  k += "}\n";
  const std::string text = "using namespace fsk;\n" + body + k;
  *entry = fmt("fs_gen_pack_%08x", fnv1a(text));
  std::string out = text;
  out.replace(out.find(kEntryPlaceholder), sizeof kEntryPlaceholder - 1, *entry);
  return out;
}

std::string embedded_prelude() { return std::string(kEmbeddedDeviceUtils) + kEmbeddedGenSupport; }

std::string generate_row_kernel(const RowProgP& p) {
  std::string s;
  s.reserve(48 * 1024);
  s += kEmbeddedDeviceUtils;
  s += kEmbeddedGenSupport;
  s += generate_row_kernel_body(p);
  return s;
}

}  // namespace fs
