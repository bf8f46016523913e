// Execution and inspection of an explored program (fs_program_*): the steps of the plan in their order, stage by
// stage where the graph names computations outside it, packed launches where the plan has them, and the joint fold
// launch behind the last step.  Nothing here allocates device memory or waits for the device.
#include <algorithm>
#include <cstring>
#include <string>

#include "fs_program.hpp"

extern "C" {
fs_status fs_pack_execute(const fs_pack* p, const void* const* inputs, void* const* outputs, void* hip_stream);

void fs_program_destroy(fs_program* p) { delete p; }

fs_status fs_program_query(const fs_program* p, fs_program_info* out) try {
  clear_error();
  if (!p || !out) return fail(FS_ERR_INVALID_ARG, "fs_program_query: null argument");
  *out = p->info;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_program_query");
}

fs_status fs_program_pattern(const fs_program* p, int32_t index, int32_t* ops, int32_t capacity, int32_t* n_ops, double* f_us,
                             int32_t* pack, fs_plan_info* info) try {
  clear_error();
  if (!p) return fail(FS_ERR_INVALID_ARG, "fs_program_pattern: null argument");
  if (index < 0 || index >= (int32_t)p->steps.size())
    return fail(FS_ERR_INVALID_ARG, "fs_program_pattern: index %d outside 0..%zu", index, p->steps.size() - 1);
  const fs_program::Step& s = p->steps[index];
  if (n_ops) *n_ops = (int32_t)s.ops.size();
  if (ops)
    for (int32_t k = 0; k < capacity && k < (int32_t)s.ops.size(); ++k) ops[k] = s.ops[k];
  if (f_us) *f_us = s.f;
  if (pack) *pack = s.pack;
  if (info) *info = s.plan->candidates[s.plan->chosen].info;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_program_pattern");
}

int64_t fs_program_describe(const fs_program* p, char* text, size_t capacity) try {
  clear_error();
  if (!p || (!text && capacity > 0)) return fail(FS_ERR_INVALID_ARG, "fs_program_describe: null argument");
  std::string s;
  char line[320];
  auto where = [](const BufRef& r) {
    char b[48];
    if (r.kind == BUF_INPUT) snprintf(b, sizeof b, "in%d", r.slot);
    else if (r.kind == BUF_OUTPUT) snprintf(b, sizeof b, "out%d", r.slot);
    else snprintf(b, sizeof b, "ws+%lld", (long long)r.offset);
    return std::string(b);
  };
  snprintf(line, sizeof line, "program steps=%zu launches=%d packs=%zu joint_fold_launches=%zu workspace=%lld\n", p->steps.size(),
           p->info.n_kernels, p->packs.size(), p->joint_folds.size(), (long long)p->info.workspace_bytes);
  s += line;
  for (size_t i = 0; i < p->steps.size(); ++i) {
    const fs_program::Step& st = p->steps[i];
    const fs_plan_info& pi = st.plan->candidates[st.plan->chosen].info;
    std::string ops;
    for (int o : st.ops) ops += (ops.empty() ? "" : ",") + std::to_string(o);
    snprintf(line, sizeof line, "step %zu ops=%s pattern=%s kernel=%s launches=%zu f_us=%.3f", i, ops.c_str(), pi.pattern, pi.kernel,
             st.pack >= 0 ? (size_t)0 : launches_issued(st.plan, st.own_launches), st.f);
    s += line;
    if (st.pack >= 0) s += " pack=" + std::to_string(st.pack);
    if (p->info.n_stages > 1) s += " stage=" + std::to_string(st.stage);
    s += "\n";
    for (size_t k = 0; k < st.in.size(); ++k) s += "  input " + std::to_string(k) + " " + where(st.in[k]) + "\n";
    for (size_t k = 0; k < st.out.size(); ++k) s += "  output " + std::to_string(k) + " " + where(st.out[k]) + "\n";
    if (pi.workspace_bytes > 0)
      s += "  scratch ws+" + std::to_string((long long)st.plan_ws_offset) + " " + std::to_string((long long)pi.workspace_bytes) + "\n";
  }
  for (size_t j = 0; j < p->packs.size(); ++j) {
    std::string members;
    for (int m : p->packs[j].steps) members += (members.empty() ? "" : ",") + std::to_string(m);
    s += "pack " + std::to_string(j) + " launches=" + std::to_string(p->packs[j].pack->info.n_kernels) + " members=" + members + "\n";
  }
  for (size_t j = 0; j < p->joint_folds.size(); ++j) {
    std::string of;
    for (const fs_program::JointFold& f : p->joint_folds[j]) of += (of.empty() ? "" : ",") + std::to_string(f.step);
    s += "joint_fold " + std::to_string(j) + " folds=" + std::to_string(p->joint_folds[j].size()) + " of_steps=" + of + "\n";
  }
  const size_t need = s.size() + 1;
  if (capacity > 0) {
    const size_t n = std::min(capacity - 1, s.size());
    memcpy(text, s.data(), n);
    text[n] = 0;
  }
  return (int64_t)need;
} catch (...) {
  return fs::fail_caught("fs_program_describe");
}

}  // extern "C"

// The steps of stages first_stage..last_stage; the joint fold launches go with the program's last stage.
static fs_status run_program(const fs_program* p, int32_t first_stage, int32_t last_stage, const void* const* inputs,
                             void* const* outputs, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || !inputs || !outputs) return fail(FS_ERR_INVALID_ARG, "fs_program_execute: null argument");
  for (int i = 0; i < p->n_inputs; ++i) {
    if (!inputs[i]) return fail(FS_ERR_INVALID_ARG, "fs_program_execute: input %d is null", i);
    if ((uintptr_t)inputs[i] & 15u) return fail(FS_ERR_ALIGN, "fs_program_execute: input %d is not 16-byte aligned", i);
  }
  for (int i = 0; i < p->n_outputs; ++i) {
    if (!outputs[i]) return fail(FS_ERR_INVALID_ARG, "fs_program_execute: output %d is null", i);
    if ((uintptr_t)outputs[i] & 15u) return fail(FS_ERR_ALIGN, "fs_program_execute: output %d is not 16-byte aligned", i);
  }
  if (p->info.workspace_bytes > 0) {
    if (!workspace || workspace_bytes < (size_t)p->info.workspace_bytes)
      return fail(FS_ERR_WORKSPACE, "fs_program_execute: workspace of %lld bytes needed, %zu given", (long long)p->info.workspace_bytes,
                  workspace_bytes);
    if ((uintptr_t)workspace & 255u) return fail(FS_ERR_ALIGN, "fs_program_execute: workspace is not 256-byte aligned");
  }
  char* ws = static_cast<char*>(workspace);
  auto address = [&](const BufRef& r) -> void* {
    if (r.kind == BUF_INPUT) return const_cast<void*>(inputs[r.slot]);
    if (r.kind == BUF_OUTPUT) return outputs[r.slot];
    return ws + r.offset;
  };
  std::vector<char> pack_done(p->packs.size(), 0);
  std::vector<const void*> in;
  std::vector<void*> out;
  for (const fs_program::Step& s : p->steps) {
    if (s.stage < first_stage || s.stage > last_stage) continue;
    if (s.pack >= 0) {
      if (pack_done[s.pack]) continue;
      pack_done[s.pack] = 1;
      in.clear();
      out.clear();
      for (int m : p->packs[s.pack].steps) {
        for (const BufRef& r : p->steps[m].in) in.push_back(address(r));
        for (const BufRef& r : p->steps[m].out) out.push_back(address(r));
      }
      const fs_status st = fs_pack_execute(p->packs[s.pack].pack, in.data(), out.data(), hip_stream);
      if (st != FS_OK) return st;
      continue;
    }
    in.clear();
    out.clear();
    for (const BufRef& r : s.in) in.push_back(address(r));
    for (const BufRef& r : s.out) out.push_back(address(r));
    const int64_t need = s.plan->candidates[s.plan->chosen].info.workspace_bytes;
    const fs_status st = run_launches(s.plan, in.data(), out.data(), need > 0 ? ws + s.plan_ws_offset : nullptr, hip_stream, s.own_launches);
    if (st != FS_OK) return st;
  }
  if (last_stage < p->info.n_stages - 1) return FS_OK;
  for (const std::vector<fs_program::JointFold>& joint : p->joint_folds) {
    FoldManyP t{};
    uint32_t blocks = 0;
    for (int k = 0; k < kFoldManyMax; ++k) t.first_block[k] = 0xffffffffu;
    for (size_t k = 0; k < joint.size(); ++k) {
      const fs_program::Step& s = p->steps[joint[k].step];
      const Launch& l = s.plan->candidates[s.plan->chosen].launches[joint[k].launch];
      void* ptr[3];
      for (int a = 0; a < 3; ++a) {
        const BufRef& r = l.ptr[a];
        ptr[a] = r.kind == BUF_INPUT ? address(s.in[r.slot]) : r.kind == BUF_OUTPUT ? address(s.out[r.slot])
                 : r.kind == BUF_WORKSPACE ? (void*)(ws + s.plan_ws_offset + r.offset) : nullptr;
      }
      const GeluP& f = l.args.u.gelu;
      t.partials[k] = static_cast<const float*>(ptr[0]);
      t.out0[k] = static_cast<float*>(ptr[1]);
      t.out1[k] = static_cast<float*>(ptr[2]);
      t.first_block[k] = blocks;
      t.n[k] = f.n_row_tiles;
      t.width[k] = f.fold_cols;
      t.stride[k] = f.cols;
      t.split[k] = f.fold_split;
      t.quads[k] = f.fold_quads;
      t.out_dt[k] = f.dt;
      blocks += l.shape.grid[0];
    }
    const int err = launch_fold_many(t, blocks, hip_stream);
    if (err != 0) return fail(FS_ERR_HIP, "fs_program_execute: launching the joint fold failed: %s", hip_error_text(err));
  }
  return FS_OK;
}

extern "C" {

fs_status fs_program_execute(const fs_program* p, const void* const* inputs, void* const* outputs, void* workspace,
                             size_t workspace_bytes, void* hip_stream) try {
  clear_error();
  if (!p) return fail(FS_ERR_INVALID_ARG, "fs_program_execute: null argument");
  return run_program(p, 0, p->info.n_stages - 1, inputs, outputs, workspace, workspace_bytes, hip_stream);
} catch (...) {
  return fs::fail_caught("fs_program_execute");
}

fs_status fs_program_execute_stage(const fs_program* p, int32_t stage, const void* const* inputs, void* const* outputs,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) try {
  clear_error();
  if (!p) return fail(FS_ERR_INVALID_ARG, "fs_program_execute_stage: null argument");
  if (stage < 0 || stage >= p->info.n_stages)
    return fail(FS_ERR_INVALID_ARG, "fs_program_execute_stage: stage %d outside 0..%d", stage, p->info.n_stages - 1);
  return run_program(p, stage, stage, inputs, outputs, workspace, workspace_bytes, hip_stream);
} catch (...) {
  return fs::fail_caught("fs_program_execute_stage");
}

}  // extern "C"
