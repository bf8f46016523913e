// Plan creation (choose scheme + launch shape by the evaluator) and execution
// (patch device pointers, enqueue the launches).  fs_execute is the only place where
// control crosses from host to device.
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <string>

#include "fs_internal.hpp"

namespace fs {

void predict(Candidate* c) {
  if (c->info.scheme == FS_SCHEME_UNFUSED) {
    // per-op plan: every launch streams its own operands and results
    const DeviceModel& d = device();
    double t = 0;
    for (const Launch& l : c->launches) {
      (void)l;
      t += d.launch_s;
    }
    t += (double)c->info.bytes_moved_model / (d.hbm_peak_Bps * d.stream_fraction);
    c->info.predicted_us = t * 1e6;
    c->info.waves_per_simd = (int32_t)d.max_waves_per_simd;
    c->info.vgprs = 0;
    return;
  }
  const Launch& l = c->launches.front();
  KernelResources res;
  if (l.kernel != K_ROW_GENERATED) {
    res = kernel_resources(l.kernel, l.args);
  } else if (l.gen) {   // compiled: the code object states its registers
    res.vgprs = gen_resources(l.gen.get()).vgprs;
    res.from_device = res.vgprs > 0;
  }
  const CostResult r = evaluate(c->cost, res.from_device ? res.vgprs : 0);
  c->info.predicted_us = r.seconds * 1e6;
  c->info.waves_per_simd = r.waves_per_simd;
  c->info.vgprs = r.vgprs;
  if (res.from_device && res.static_lds > c->info.lds_bytes) c->info.lds_bytes = res.static_lds;
}

// the choice among candidates: a fallback only when nothing else stands, otherwise the lower estimate
static bool preferred(const Candidate& a, const Candidate& b) {
  if (a.fallback != b.fallback) return !a.fallback;
  return a.info.predicted_us < b.info.predicted_us;
}

static bool satisfies(const fs_plan_info& i, const fs_plan_opts& o) {
  if (o.block_threads > 0 && i.block[0] != o.block_threads) return false;
  if (o.lanes_per_row > 0 && i.lanes_per_row != o.lanes_per_row) return false;
  if (o.vecs_per_lane > 0 && i.vecs_per_lane != o.vecs_per_lane) return false;
  return true;
}

namespace {
std::atomic<int> g_codegen{-1};   // -1: not decided yet (the environment decides at first use)
}

bool codegen_enabled() {
  int v = g_codegen.load(std::memory_order_relaxed);
  if (v < 0) {
    const char* e = getenv("FS_CODEGEN");
    v = (e && e[0] == '0') ? 0 : 1;
    g_codegen.store(v, std::memory_order_relaxed);
  }
  return v != 0 && gen_available();
}

// The pattern as a row program with a launch shape, for packed launches generated over several plans: the chosen
// candidate's own program if it runs one, else (a hand-written family) the best generated shape of the same pattern.
// Patterns with column sums stay out: their fold is a launch of its own.
static void fill_generic_form(const fs_graph& g, fs_plan* p) {
  auto take = [&](const Candidate& c) {
    if (c.launches.size() != 1) return false;
    const Launch& l = c.launches.front();
    if ((l.kernel != K_ROW_GENERATED && l.kernel != K_ROW_PROGRAM) || l.args.u.prog.n_colsum > 0) return false;
    if (l.shape.block[0] != 256) return false;   // a packed kernel's workgroups have 256 threads
    if (l.args.u.prog.col_chunks > 1) return false;   // rows worked through in chunks: a launch of its own
    p->generic.valid = true;
    p->generic.prog = l.args.u.prog;
    for (int k = 0; k < kMaxPtrs; ++k) p->generic.ptr[k] = l.ptr[k];
    p->generic.blocks = l.shape.grid[0];
    return true;
  };
  if (take(p->candidates[p->chosen])) return;
  if (p->candidates[p->chosen].info.scheme == FS_SCHEME_UNFUSED) return;
  std::vector<Candidate> cands;
  if (!build_row_program(g, &cands)) return;
  int best = -1;
  for (int i = 0; i < (int)cands.size(); ++i) {
    if (cands[i].launches.size() != 1 || cands[i].launches.front().kernel != K_ROW_GENERATED) continue;
    if (cands[i].launches.front().shape.block[0] != 256 || cands[i].launches.front().args.u.prog.col_chunks > 1) continue;
    predict(&cands[i]);
    if (best < 0 || cands[i].info.predicted_us < cands[best].info.predicted_us) best = i;
  }
  if (best >= 0) take(cands[best]);
}

fs_status complete_plan(fs_plan* p) {
  const fs_plan_opts& o = p->opts;
  for (;;) {
    Candidate& c = p->candidates[p->chosen];
    Launch* gen = nullptr;
    for (Launch& l : c.launches)
      if (l.kernel == K_ROW_GENERATED && !l.gen) gen = &l;
    if (!gen) return FS_OK;
    std::string log;
    const int err = gen_compile(generate_row_kernel(gen->args.u.prog), generated_kernel_entry(gen->args.u.prog).c_str(), &gen->gen, &log);
    bool usable = err == 0;
    std::string why;
    if (!usable) {
      why = "compiling the generated kernel failed: " + log;
    } else {
      const GenResources res = gen_resources(gen->gen.get());
      if (res.scratch_bytes > 0) {   // values spilled to per-lane scratch memory: the shape holds too much per lane
        usable = false;
        why = "the generated kernel keeps " + std::to_string(res.scratch_bytes) + " bytes per lane in scratch memory";
      }
    }
    if (usable) {
      const int e = gen_preload(gen->gen.get());
      if (e != 0) return fail(FS_ERR_HIP, "fs_plan_create: loading the generated kernel failed: %s", hip_error_text(e));
      predict(&c);   // with the compiled kernel's own register count
      return FS_OK;
    }
    gen->gen.reset();
    if (o.candidate >= 0) return fail(FS_ERR_UNSUPPORTED_PATTERN, "fs_plan_create: candidate %d: %s", o.candidate, why.c_str());
    // this candidate is out; take the best of the rest
    c.info.predicted_us = 1e30;
    int best = -1;
    for (int i = 0; i < (int)p->candidates.size(); ++i) {
      const Candidate& k = p->candidates[i];
      if (k.info.predicted_us >= 1e30 || !satisfies(k.info, o)) continue;
      if (best < 0 || preferred(k, p->candidates[best])) best = i;
    }
    if (best < 0) return fail(FS_ERR_UNSUPPORTED_PATTERN, "fs_plan_create: %s, and no other candidate has the requested launch shape", why.c_str());
    p->chosen = best;
  }
}

}  // namespace fs

using namespace fs;

size_t fs::launches_issued(const fs_plan* p, size_t n_launches) {
  const Candidate& c = p->candidates[p->chosen];
  const size_t end = std::min(n_launches, c.launches.size());
  size_t issued = 0;
  for (size_t li = 0; li < end; ++li, ++issued)
    if (c.launches[li].kernel == K_COLFOLD)
      for (size_t folds = 1; li + 1 < end && folds < (size_t)kFoldManyMax && c.launches[li + 1].kernel == K_COLFOLD; ++folds) ++li;
  return issued;
}

fs_status fs::run_launches(const fs_plan* p, const void* const* inputs, void* const* outputs, void* workspace, void* hip_stream,
                       size_t n_launches) {
  const Candidate& c = p->candidates[p->chosen];
  const size_t end = std::min(n_launches, c.launches.size());
  auto address = [&](const BufRef& r) -> void* {
    switch (r.kind) {
      case BUF_INPUT: return const_cast<void*>(inputs[r.slot]);
      case BUF_OUTPUT: return outputs[r.slot];
      case BUF_WORKSPACE: return static_cast<char*>(workspace) + r.offset;
      default: return nullptr;
    }
  };
  for (size_t li = 0; li < end; ++li) {
    const Launch& l = c.launches[li];
    // several folds of column partial sums in a row (a pattern with more than two column sums, or sums of different
    // dtypes) are independent of each other: they go out as one launch
    size_t folds = 0;
    while (li + folds < end && folds < (size_t)kFoldManyMax && c.launches[li + folds].kernel == K_COLFOLD) ++folds;
    if (folds >= 2) {
      FoldManyP t{};
      uint32_t blocks = 0;
      for (int k = 0; k < kFoldManyMax; ++k) t.first_block[k] = 0xffffffffu;
      for (size_t k = 0; k < folds; ++k) {
        const Launch& f = c.launches[li + k];
        const GeluP& fp = f.args.u.gelu;
        t.partials[k] = static_cast<const float*>(address(f.ptr[0]));
        t.out0[k] = static_cast<float*>(address(f.ptr[1]));
        t.out1[k] = static_cast<float*>(address(f.ptr[2]));
        t.first_block[k] = blocks;
        t.n[k] = fp.n_row_tiles;
        t.width[k] = fp.fold_cols;
        t.stride[k] = fp.cols;
        t.split[k] = fp.fold_split;
        t.quads[k] = fp.fold_quads;
        t.out_dt[k] = fp.dt;
        blocks += f.shape.grid[0];
      }
      const int err = launch_fold_many(t, blocks, hip_stream);
      if (err != 0) return fail(FS_ERR_HIP, "fs_execute: launching the folds failed: %s", hip_error_text(err));
      li += folds - 1;
      continue;
    }
    KernelArgs a = l.args;
    for (int k = 0; k < kMaxPtrs; ++k) a.p[k] = address(l.ptr[k]);
    int err;
    if (l.kernel == K_ROW_GENERATED) {
      if (!l.gen) return fail(FS_ERR_INVALID_ARG, "fs_execute: the plan's generated kernel was never compiled");
      err = gen_launch(l.gen.get(), a.p, sizeof(void*) * kGenArgPtrs, l.shape, hip_stream);
    } else {
      err = launch_kernel(l.kernel, a, l.shape, hip_stream);
    }
    if (err != 0) return fail(FS_ERR_HIP, "fs_execute: launching %s failed: %s", kernel_name(l.kernel), hip_error_text(err));
  }
  return FS_OK;
}

fs_status fs::check_execute_args(const fs_plan* p, const void* const* inputs, void* const* outputs, const char* who) {
  if (!p || !inputs || !outputs) return fail(FS_ERR_INVALID_ARG, "%s: null argument", who);
  for (int i = 0; i < p->n_inputs; ++i) {
    if (!inputs[i]) return fail(FS_ERR_INVALID_ARG, "%s: input %d is null", who, i);
    if ((uintptr_t)inputs[i] & 15u) return fail(FS_ERR_ALIGN, "%s: input %d is not 16-byte aligned", who, i);
  }
  for (int i = 0; i < p->n_outputs; ++i) {
    if (!outputs[i]) return fail(FS_ERR_INVALID_ARG, "%s: output %d is null", who, i);
    if ((uintptr_t)outputs[i] & 15u) return fail(FS_ERR_ALIGN, "%s: output %d is not 16-byte aligned", who, i);
  }
  return FS_OK;
}

fs_status fs::create_plan(const fs_graph* g, int32_t scheme, const fs_plan_opts* opts, bool complete, fs_plan** out) {
  if (!g || !out) return fail(FS_ERR_INVALID_ARG, "fs_plan_create: null argument");
  if (!g->finalized) return fail(FS_ERR_INVALID_ARG, "fs_plan_create: graph is not finalized");
  if (!g->external.empty())
    return fail(FS_ERR_UNSUPPORTED_PATTERN, "fs_plan_create: the graph waits for external computations between its ops; no single plan runs it (use fs_explore)");
  if (scheme < FS_SCHEME_AUTO || scheme > FS_SCHEME_GLOBAL) return fail(FS_ERR_INVALID_ARG, "fs_plan_create: bad scheme %d", scheme);
  fs_plan_opts o = {-1, 0, 0, 0};
  if (opts) {
    o = *opts;
    // the public field counts from 1 (0 = choose, so a zero-initialised struct asks for nothing); inside, -1 = choose
    o.candidate = opts->candidate > 0 ? opts->candidate - 1 : -1;
  }

  std::vector<Candidate> all;
  std::string pattern;
  PackForm pack_form;
  if (scheme != FS_SCHEME_UNFUSED) {
    pattern = build_stitched(*g, &all, &pack_form);
    for (Candidate& c : all) predict(&c);
  }
  if (scheme == FS_SCHEME_UNFUSED || (scheme == FS_SCHEME_AUTO && all.empty())) {
    Candidate u;
    const fs_status s = build_unfused(*g, &u);
    if (s != FS_OK) return s;
    predict(&u);
    all.clear();
    all.push_back(u);
  } else if (all.empty()) {
    if (pattern.empty())
      return fail(FS_ERR_UNSUPPORTED_PATTERN, "fs_plan_create: no stitched kernel matches this graph (scheme %s)", scheme_name(scheme));
    return fail(FS_ERR_UNSUPPORTED_PATTERN,
                "fs_plan_create: pattern '%s' recognised, but its shapes / dtypes fit no stitched kernel", pattern.c_str());
  }

  // keep the candidates of the requested scheme; AUTO keeps all of them
  std::vector<Candidate> kept;
  for (const Candidate& c : all)
    if (scheme == FS_SCHEME_AUTO || scheme == FS_SCHEME_UNFUSED || c.info.scheme == scheme) kept.push_back(c);
  if (kept.empty())
    return fail(FS_ERR_LOCALITY,
                "fs_plan_create: pattern '%s' has no %s schedule that keeps its reduction rows inside the reuse scope",
                pattern.c_str(), scheme_name(scheme));

  int best = -1;
  if (o.candidate >= 0) {
    if (o.candidate >= (int32_t)kept.size())
      return fail(FS_ERR_INVALID_ARG, "fs_plan_create: candidate %d outside 0..%zu", o.candidate, kept.size() - 1);
    best = o.candidate;
  } else {
    for (int i = 0; i < (int)kept.size(); ++i) {
      if (!satisfies(kept[i].info, o)) continue;
      if (best < 0 || preferred(kept[i], kept[best])) best = i;
    }
    if (best < 0)
      return fail(FS_ERR_LOCALITY, "fs_plan_create: no %s candidate of pattern '%s' has the requested launch shape",
                  scheme_name(scheme), pattern.c_str());
  }

  fs_plan* p = new (std::nothrow) fs_plan();
  if (!p) return fail(FS_ERR_INVALID_ARG, "fs_plan_create: out of host memory");
  p->candidates = kept;
  p->chosen = best;
  for (size_t i = 0; i < p->candidates.size(); ++i) {
    p->candidates[i].info.n_candidates = (int32_t)p->candidates.size();
    p->candidates[i].info.candidate = (int32_t)i;
  }
  p->pack = pack_form;
  p->opts = o;
  p->bytes_min = graph_bytes_min(*g);
  p->n_inputs = (int32_t)g->inputs.size();
  p->n_outputs = (int32_t)g->outputs.size();
  for (int t : g->inputs) p->input_bytes.push_back(g->tensors[t].numel() * dtype_bytes(g->tensors[t].dtype));
  for (int t : g->outputs) p->output_bytes.push_back(g->tensors[t].numel() * dtype_bytes(g->tensors[t].store_as));
  if (scheme != FS_SCHEME_UNFUSED && codegen_enabled()) fill_generic_form(*g, p);
  if (complete) {
    const fs_status s = complete_plan(p);
    if (s != FS_OK) {
      delete p;
      // AUTO promises a plan for every valid graph: when the only stitched form was a generated kernel and that
      // did not compile, the per-op plan is what remains
      if (scheme == FS_SCHEME_AUTO && o.candidate < 0 && s == FS_ERR_UNSUPPORTED_PATTERN) {
        fs_plan_opts plain = o;
        plain.candidate = 0;
        return create_plan(g, FS_SCHEME_UNFUSED, &plain, true, out);
      }
      return s;
    }
  }
  *out = p;
  return FS_OK;
}

extern "C" {

fs_status fs_plan_create(const fs_graph* g, int32_t scheme, const fs_plan_opts* opts, fs_plan** out) try {
  clear_error();
  return create_plan(g, scheme, opts, true, out);
} catch (...) {
  return fs::fail_caught("fs_plan_create");
}

int32_t fs_codegen_enable(int32_t on) try {
  const int32_t before = codegen_enabled() ? 1 : 0;
  g_codegen.store(on ? 1 : 0, std::memory_order_relaxed);
  return before;
} catch (...) {
  return fs::fail_caught("fs_codegen_enable");
}

int32_t fs_codegen_available(void) { return gen_available() ? 1 : 0; }

void fs_plan_destroy(fs_plan* p) { delete p; }

fs_status fs_plan_query(const fs_plan* p, fs_plan_info* out) try {
  clear_error();
  if (!p || !out) return fail(FS_ERR_INVALID_ARG, "fs_plan_query: null argument");
  *out = p->candidates[p->chosen].info;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_plan_query");
}

fs_status fs_plan_candidate(const fs_plan* p, int32_t index, fs_plan_info* out) try {
  clear_error();
  if (!p || !out) return fail(FS_ERR_INVALID_ARG, "fs_plan_candidate: null argument");
  if (index < 0 || index >= (int32_t)p->candidates.size())
    return fail(FS_ERR_INVALID_ARG, "fs_plan_candidate: index %d outside 0..%zu", index, p->candidates.size() - 1);
  *out = p->candidates[index].info;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_plan_candidate");
}

int64_t fs_plan_describe(const fs_plan* p, char* text, size_t capacity) try {
  clear_error();
  if (!p || (!text && capacity > 0)) return fail(FS_ERR_INVALID_ARG, "fs_plan_describe: null argument");
  const Candidate& c = p->candidates[p->chosen];
  std::string s;
  char line[256];
  auto buf_name = [&](const BufRef& r) {
    char b[48];
    if (r.kind == BUF_INPUT) snprintf(b, sizeof b, "in%d", r.slot);
    else if (r.kind == BUF_OUTPUT) snprintf(b, sizeof b, "out%d", r.slot);
    else if (r.kind == BUF_WORKSPACE) snprintf(b, sizeof b, "ws+%lld", (long long)r.offset);
    else snprintf(b, sizeof b, "-");
    return std::string(b);
  };
  snprintf(line, sizeof line, "plan pattern=%s scheme=%s launches=%zu\n", c.info.pattern, scheme_name(c.info.scheme), launches_issued(p, c.launches.size()));
  s += line;
  for (const Launch& l : c.launches) {
    snprintf(line, sizeof line, "launch %s grid=%u block=%u lds=%u\n", kernel_name(l.kernel), l.shape.grid[0] * l.shape.grid[1] * l.shape.grid[2],
             l.shape.block[0] * l.shape.block[1] * l.shape.block[2], l.shape.lds_bytes);
    s += line;
    if (l.kernel == K_ROW_GENERATED) s += "  entry " + generated_kernel_entry(l.args.u.prog) + "\n";
    if (l.kernel != K_ROW_PROGRAM && l.kernel != K_ROW_GENERATED) {
      for (int k = 0; k < kMaxPtrs; ++k)
        if (l.ptr[k].kind != BUF_NONE) s += "  ptr" + std::to_string(k) + " " + buf_name(l.ptr[k]) + "\n";
      continue;
    }
    const RowProgP& q = l.args.u.prog;
    snprintf(line, sizeof line, "  program vec=%d rows=%u cols=%u lanes=%d vecs=%d regs=%d sregs=%d lead=%u,%u,%u\n", q.vec, q.rows, q.cols,
             q.lanes_per_row, q.vecs_per_lane, q.n_regs, q.n_sregs, q.od[0].d, q.od[1].d, q.od[2].d);
    s += line;
    for (int i = 0; i < q.n_full; ++i)
      s += "  full " + buf_name(l.ptr[i]) + " reg " + std::to_string(q.full_reg[i]) + " " + dtype_name(q.full_dt[i]) +
           (((q.full_bcast >> i) & 1u) ? " rowstrides=" + std::to_string(q.ms[i][0]) + "," + std::to_string(q.ms[i][1]) + "," +
                                             std::to_string(q.ms[i][2]) : std::string()) +
           (q.acc_input == i ? " acc" : "") + "\n";
    for (int i = 0; i < q.n_col; ++i)
      s += "  col " + buf_name(l.ptr[kSlotCol + i]) + " index " + std::to_string(i) + " " + dtype_name(q.col_dt[i]) + "\n";
    for (int i = 0; i < q.n_rscal; ++i)
      s += "  rscal " + buf_name(l.ptr[kSlotRscal + i]) + " sreg " + std::to_string(q.rscal_sreg[i]) + " " + dtype_name(q.rscal_dt[i]) +
           (((q.rscal_bcast >> i) & 1u) ? " rowstrides=" + std::to_string(q.rms[i][0]) + "," + std::to_string(q.rms[i][1]) + "," +
                                              std::to_string(q.rms[i][2]) : std::string()) + "\n";
    for (int i = 0; i < kProgMaxOperands; ++i)
      if (l.ptr[kSlotOut + i].kind != BUF_NONE)
        s += "  output " + std::to_string(i) + " " + buf_name(l.ptr[kSlotOut + i]) +
             (((q.out_perm >> i) & 1u) ? " rowstrides=" + std::to_string(q.oms[i][0]) + "," + std::to_string(q.oms[i][1]) + "," +
                                            std::to_string(q.oms[i][2]) : std::string()) + "\n";
    for (int i = 0; i < kProgMaxOperands; ++i)
      if (l.ptr[kSlotRout + i].kind != BUF_NONE) s += "  routput " + std::to_string(i) + " " + buf_name(l.ptr[kSlotRout + i]) + "\n";
    if (q.n_colsum > 0)   // partial sums: one row of n_colsum * cols floats per workgroup, folded by the next launch
      s += "  colsums " + std::to_string(q.n_colsum) + " partials " + buf_name(l.ptr[kSlotWs]) + " rows_per_group " +
           std::to_string(q.rows_per_group) + " col_tiles " + std::to_string(q.col_tiles > 1 ? q.col_tiles : 1) + "\n";
    if (q.col_chunks > 1)   // the row in pieces of lanes * vecs steps, a pass per row reduction and one for the stores
      s += "  chunks " + std::to_string(q.col_chunks) + " of " + std::to_string(q.lanes_per_row * q.vecs_per_lane * q.vec) + " columns" +
           (q.col_kept > 0 ? ", the first " + std::to_string(q.col_kept) + " kept in registers" : std::string()) + "\n";
    static const char* op_names[] = {"add", "sub", "rsub", "mul", "div", "rdiv", "max", "square", "exp", "rsqrt", "tanh", "gelu",
                                     "gelu_grad", "log", "sigmoid", "relu", "abs", "sqrt", "cvt", "load", "rsum", "rmax", "rsumsq", "store", "store_scal", "colsum"};
    static const char* kind_names[] = {"acc", "sacc", "reg", "scal", "imm", "col"};
    for (int i = 0; i < q.n_instr; ++i) {
      const ProgInstr& in = q.instr[i];
      snprintf(line, sizeof line, "  instr %d %s b=%s:%d dst=%d flags=%s%s aux=%d imm=%.9g\n", i, op_names[in.op], kind_names[in.b_kind],
               in.b, in.dst, (in.flags & PF_SCALAR) ? "s" : "v", (in.flags & PF_KEEP) ? "k" : "-", in.aux, (double)in.imm);
      s += line;
    }
  }
  if (capacity > 0) {
    const size_t n = std::min(capacity - 1, s.size());
    memcpy(text, s.data(), n);
    text[n] = 0;
  }
  return (int64_t)s.size() + 1;
} catch (...) {
  return fs::fail_caught("fs_plan_describe");
}

int64_t fs_plan_source(const fs_plan* p, char* text, size_t capacity) try {
  clear_error();
  if (!p || (!text && capacity > 0)) return fail(FS_ERR_INVALID_ARG, "fs_plan_source: null argument");
  std::string s;
  for (const Launch& l : p->candidates[p->chosen].launches)
    if (l.kernel == K_ROW_GENERATED) s += generate_row_kernel_body(l.args.u.prog);
  if (capacity > 0) {
    const size_t n = std::min(capacity - 1, s.size());
    memcpy(text, s.data(), n);
    text[n] = 0;
  }
  return (int64_t)s.size() + 1;
} catch (...) {
  return fs::fail_caught("fs_plan_source");
}

fs_status fs_execute(const fs_plan* p, const void* const* inputs, void* const* outputs, void* workspace,
                     size_t workspace_bytes, void* hip_stream) try {
  clear_error();
  const fs_status s = check_execute_args(p, inputs, outputs, "fs_execute");
  if (s != FS_OK) return s;
  const Candidate& c = p->candidates[p->chosen];
  if (c.info.workspace_bytes > 0) {
    if (!workspace || workspace_bytes < (size_t)c.info.workspace_bytes)
      return fail(FS_ERR_WORKSPACE, "fs_execute: workspace of %lld bytes needed, %zu given", (long long)c.info.workspace_bytes, workspace_bytes);
    if ((uintptr_t)workspace & 15u) return fail(FS_ERR_ALIGN, "fs_execute: workspace is not 16-byte aligned");
  }
  return run_launches(p, inputs, outputs, workspace, hip_stream, c.launches.size());
} catch (...) {
  return fs::fail_caught("fs_execute");
}

fs_status fs_stream_copy(void* dst, const void* src, size_t bytes, void* hip_stream) try {
  clear_error();
  if (!dst || !src) return fail(FS_ERR_INVALID_ARG, "fs_stream_copy: null pointer");
  if (((uintptr_t)dst | (uintptr_t)src | bytes) & 15u) return fail(FS_ERR_ALIGN, "fs_stream_copy: pointers and size must be multiples of 16");
  if (bytes == 0) return FS_OK;
  if (bytes / 16 >= (size_t(1) << 32)) return fail(FS_ERR_SHAPE, "fs_stream_copy: too large");
  KernelArgs a;
  a.p[0] = const_cast<void*>(src);
  a.p[1] = dst;
  a.u.unary = UnaryP{};
  a.u.unary.n = (uint32_t)(bytes / 16);
  LaunchShape s;
  s.block[0] = 256;
  s.grid[0] = (uint32_t)((bytes / 16 + 1023) / 1024);
  const int err = launch_kernel(K_COPY, a, s, hip_stream);
  if (err != 0) return fail(FS_ERR_HIP, "fs_stream_copy: %s", hip_error_text(err));
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_stream_copy");
}

}  // extern "C"
