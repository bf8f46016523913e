// Packed execution: several independent fusion patterns in one launch (kernel packing,
// paper Section 4.1, applied across patterns as in remote fusion, Section 5.3).  A pack
// is built from finished plans; each member contributes the packed form its pattern
// matcher recorded.  Execution fills the operand pointers into a table that travels in
// the kernel arguments, so nothing is allocated or copied on the device side.
#include <algorithm>
#include <cstring>

#include "fs_internal.hpp"

namespace fs {
namespace {

int types_of(const PackForm& f) {
  if (f.in_dt == f.out_dt) {
    if (f.in_dt == FS_F32) return PT_F32;
    if (f.in_dt == FS_F16) return PT_F16;
    if (f.in_dt == FS_BF16) return PT_BF16;
    return -1;
  }
  if (f.in_dt == FS_F32 && f.out_dt == FS_BF16 && (f.spec == PACK_LN_FULL || f.spec == PACK_LN_PLAIN)) return PT_F32_BF16;
  return -1;
}

// lanes per row and vectors per lane for a member: a lane group of a wavefront while the
// row fits 64 lanes x 4 vectors, else the whole 256-thread workgroup
bool shape_member(const PackForm& f, PackEntry* e, uint32_t* blocks) {
  const uint32_t vec = 16u / (uint32_t)dtype_bytes(f.in_dt);
  if (f.cols == 0 || f.rows == 0 || f.cols % vec != 0) return false;
  const uint32_t nvec = f.cols / vec;
  uint32_t L, K;
  if (nvec <= 256) {
    K = nvec <= 64 ? 1 : (nvec <= 128 ? 2 : 4);
    L = 1;
    while (L * K < nvec) L <<= 1;
    *blocks = (f.rows + 256 / L - 1) / (256 / L);
  } else if (nvec <= 1024) {
    K = nvec <= 512 ? 2 : 4;
    L = 256;
    *blocks = f.rows;
  } else {
    return false;
  }
  e->p = RowP{};
  e->p.pattern = f.spec;
  e->p.dt = f.in_dt;
  e->p.rows = f.rows;
  e->p.cols = f.cols;
  for (int i = 0; i < 4; ++i) e->p.f[i] = f.f[i];
  e->p.lanes_per_row = (int32_t)L;
  int lg = 0;
  while ((1u << lg) < L) ++lg;
  e->p.lanes_log2 = lg;
  e->p.vecs_per_lane = (int32_t)K;
  e->p.fast = 0;
  const int k_log2 = K == 1 ? 0 : (K == 2 ? 1 : 2);
  e->variant = (f.spec * PT_COUNT + types_of(f)) * 3 + k_log2;
  return true;
}

// The pack as generated kernels, one per 32 members, each made for exactly its members (a device function per
// member, dispatched on the workgroup index; the operand pointers travel in one table in the kernel arguments).
// false if some member has no row-program form or a kernel does not compile: the caller then tries the fixed
// packed kernel.
bool build_generated_pack(const fs_plan* const* plans, int32_t n, fs_pack* pk) {
  if (!codegen_enabled()) return false;
  for (int i = 0; i < n; ++i)
    if (!plans[i] || !plans[i]->generic.valid) return false;
  int32_t first_input = 0, first_output = 0;
  int32_t vgprs = 0;
  for (int begin = 0; begin < n; begin += kPackMaxMembers) {
    const int end = std::min(n, begin + kPackMaxMembers);
    std::vector<RowProgP> progs;
    std::vector<uint32_t> blocks;
    uint64_t total = 0;
    for (int i = begin; i < end; ++i) {
      progs.push_back(plans[i]->generic.prog);
      blocks.push_back(plans[i]->generic.blocks);
      total += plans[i]->generic.blocks;
    }
    if (total >= (1ull << 31)) return false;
    std::vector<std::vector<int>> slots;
    std::string entry;
    const std::string source = embedded_prelude() + generate_pack_kernel(progs, blocks, &slots, &entry);
    fs_pack::GenLaunch gl;
    std::string log;
    if (gen_compile(source, entry.c_str(), &gl.kernel, &log) != 0) return false;
    const GenResources res = gen_resources(gl.kernel.get());
    if (res.scratch_bytes > 0) return false;
    if (gen_preload(gl.kernel.get()) != 0) return false;
    vgprs = std::max(vgprs, res.vgprs);
    gl.blocks = (uint32_t)total;
    for (int i = begin; i < end; ++i) {
      const fs_plan* p = plans[i];
      for (int slot : slots[i - begin]) {
        const BufRef& r = p->generic.ptr[slot];
        fs_pack::PtrRef pr;
        pr.kind = r.kind;
        pr.index = (r.kind == BUF_INPUT ? first_input : first_output) + r.slot;
        if (r.kind != BUF_INPUT && r.kind != BUF_OUTPUT) return false;
        gl.ptrs.push_back(pr);
      }
      first_input += p->n_inputs;
      first_output += p->n_outputs;
    }
    if (gl.ptrs.size() > 480) return false;   // the table travels in 4 KB of kernel arguments
    pk->info.grid += (int32_t)total;
    pk->generated.push_back(gl);
  }
  pk->info.vgprs = vgprs;
  return true;
}

}  // namespace
}  // namespace fs

using namespace fs;

extern "C" {

fs_status fs_pack_create(const fs_plan* const* plans, int32_t n, fs_pack** out) try {
  clear_error();
  if (!plans || !out) return fail(FS_ERR_INVALID_ARG, "fs_pack_create: null argument");
  if (n < 1 || n > FS_PACK_MAX_MEMBERS) return fail(FS_ERR_INVALID_ARG, "fs_pack_create: %d members, 1..%d allowed", n, FS_PACK_MAX_MEMBERS);
  fs_pack* pk = new (std::nothrow) fs_pack();
  if (!pk) return fail(FS_ERR_INVALID_ARG, "fs_pack_create: out of host memory");
  double separate_us = 0, body_s = 0;
  int64_t bytes = 0;
  for (int i = 0; i < n; ++i)
    if (!plans[i]) { delete pk; return fail(FS_ERR_INVALID_ARG, "fs_pack_create: plan %d is null", i); }
  if (build_generated_pack(plans, n, pk)) {
    const DeviceModel& dm = device();
    for (int i = 0; i < n; ++i) {
      fs_pack::Member m;
      m.first_input = pk->n_inputs;
      m.n_inputs = plans[i]->n_inputs;
      m.first_output = pk->n_outputs;
      pk->n_inputs += plans[i]->n_inputs;
      pk->n_outputs += plans[i]->n_outputs;
      pk->members.push_back(m);
      separate_us += plans[i]->candidates[plans[i]->chosen].info.predicted_us;
      bytes += plans[i]->bytes_min;
    }
    body_s = std::max((double)bytes / (dm.hbm_peak_Bps * dm.stream_fraction), dm.mem_latency_s * 2);
    pk->info.n_members = n;
    pk->info.n_kernels = (int32_t)pk->generated.size();
    pk->info.block = 256;
    pk->info.n_inputs = pk->n_inputs;
    pk->info.n_outputs = pk->n_outputs;
    pk->info.bytes_min = bytes;
    pk->info.predicted_us = (dm.launch_s * pk->info.n_kernels + body_s) * 1e6;
    pk->info.predicted_separate_us = separate_us;
    pk->info.generated = 1;
    *out = pk;
    return FS_OK;
  }
  pk->generated.clear();
  pk->info = fs_pack_info{};
  auto empty_table = [] {
    PackTable t{};
    for (uint32_t& fb : t.first_block) fb = 0xFFFFFFFFu;
    return t;
  };
  PackTable cur = empty_table();
  uint64_t total_blocks = 0;
  const DeviceModel& d = device();
  for (int i = 0; i < n; ++i) {
    const fs_plan* p = plans[i];
    if (!p) { delete pk; return fail(FS_ERR_INVALID_ARG, "fs_pack_create: plan %d is null", i); }
    if (p->pack.spec < 0 || types_of(p->pack) < 0) {
      delete pk;
      return fail(FS_ERR_UNSUPPORTED_PATTERN, "fs_pack_create: plan %d (pattern '%s') has no packed form", i,
                  p->candidates[p->chosen].info.pattern);
    }
    PackEntry e{};
    uint32_t blocks = 0;
    if (!shape_member(p->pack, &e, &blocks)) {
      delete pk;
      return fail(FS_ERR_LOCALITY, "fs_pack_create: plan %d: a row of %u elements does not fit one workgroup's registers", i, p->pack.cols);
    }
    if (cur.n == kPackMaxMembers) {
      cur.total_blocks = (uint32_t)total_blocks;
      pk->tables.push_back(cur);
      cur = empty_table();
      total_blocks = 0;
    }
    cur.first_block[cur.n] = (uint32_t)total_blocks;
    total_blocks += blocks;
    if (total_blocks >= (1ull << 31)) { delete pk; return fail(FS_ERR_SHAPE, "fs_pack_create: too many workgroups"); }
    cur.e[cur.n++] = e;
    fs_pack::Member m;
    m.form = p->pack;
    m.first_input = pk->n_inputs;
    m.n_inputs = p->n_inputs;
    m.first_output = pk->n_outputs;
    pk->n_inputs += p->n_inputs;
    pk->n_outputs += p->n_outputs;
    pk->members.push_back(m);
    separate_us += p->candidates[p->chosen].info.predicted_us;
    bytes += p->bytes_min;
    pk->info.grid += (int32_t)blocks;
  }
  cur.total_blocks = (uint32_t)total_blocks;
  pk->tables.push_back(cur);
  // one launch plus the members' bytes at the streaming rate; members too small to fill
  // the device still pay one memory round trip
  body_s = std::max((double)bytes / (d.hbm_peak_Bps * d.stream_fraction), d.mem_latency_s * 2);
  pk->info.n_members = n;
  pk->info.n_kernels = (int32_t)pk->tables.size();
  pk->info.block = 256;
  pk->info.n_inputs = pk->n_inputs;
  pk->info.n_outputs = pk->n_outputs;
  pk->info.bytes_min = bytes;
  pk->info.predicted_us = (d.launch_s * pk->info.n_kernels + body_s) * 1e6;
  pk->info.predicted_separate_us = separate_us;
  const KernelResources r = pack_kernel_resources();
  pk->info.vgprs = r.from_device ? r.vgprs : 0;
  *out = pk;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_pack_create");
}

void fs_pack_destroy(fs_pack* p) { delete p; }

fs_status fs_pack_query(const fs_pack* p, fs_pack_info* out) try {
  clear_error();
  if (!p || !out) return fail(FS_ERR_INVALID_ARG, "fs_pack_query: null argument");
  *out = p->info;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_pack_query");
}

fs_status fs_pack_execute(const fs_pack* p, const void* const* inputs, void* const* outputs, void* hip_stream) try {
  clear_error();
  if (!p || !inputs || !outputs) return fail(FS_ERR_INVALID_ARG, "fs_pack_execute: null argument");
  for (int i = 0; i < p->n_inputs; ++i) {
    if (!inputs[i]) return fail(FS_ERR_INVALID_ARG, "fs_pack_execute: input %d is null", i);
    if ((uintptr_t)inputs[i] & 15u) return fail(FS_ERR_ALIGN, "fs_pack_execute: input %d is not 16-byte aligned", i);
  }
  for (int i = 0; i < p->n_outputs; ++i) {
    if (!outputs[i]) return fail(FS_ERR_INVALID_ARG, "fs_pack_execute: output %d is null", i);
    if ((uintptr_t)outputs[i] & 15u) return fail(FS_ERR_ALIGN, "fs_pack_execute: output %d is not 16-byte aligned", i);
  }
  for (const fs_pack::GenLaunch& gl : p->generated) {
    void* table[512];
    for (size_t k = 0; k < gl.ptrs.size(); ++k)
      table[k] = gl.ptrs[k].kind == BUF_INPUT ? const_cast<void*>(inputs[gl.ptrs[k].index]) : outputs[gl.ptrs[k].index];
    LaunchShape shape;
    shape.grid[0] = gl.blocks;
    shape.block[0] = 256;
    const int err = gen_launch(gl.kernel.get(), table, sizeof(void*) * std::max<size_t>(gl.ptrs.size(), 1), shape, hip_stream);
    if (err != 0) return fail(FS_ERR_HIP, "fs_pack_execute: launching the generated packed kernel failed: %s", hip_error_text(err));
  }
  if (!p->generated.empty()) return FS_OK;
  size_t m = 0;
  for (const PackTable& tpl : p->tables) {
    PackTable t = tpl;
    for (int k = 0; k < t.n; ++k, ++m) {
      const fs_pack::Member& mem = p->members[m];
      PackEntry& e = t.e[k];
      for (int i = 0; i < 2; ++i) e.in[i] = mem.form.in_slot[i] >= 0 ? inputs[mem.first_input + mem.form.in_slot[i]] : nullptr;
      for (int i = 0; i < 3; ++i) e.vec[i] = mem.form.vec_slot[i] >= 0 ? inputs[mem.first_input + mem.form.vec_slot[i]] : nullptr;
      e.out = outputs[mem.first_output];
    }
    const int err = launch_pack(t, hip_stream);
    if (err != 0) return fail(FS_ERR_HIP, "fs_pack_execute: launching the packed kernel failed: %s", hip_error_text(err));
  }
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_pack_execute");
}

}  // extern "C"
