// TEST-ONLY stand-in for kernels/*.hip: lets the host core (graph, matcher, evaluator, planner, explorer, row-program
// compiler, code generator, executor) be built with the host compiler and its sanitizers and "executed" on a machine
// without a GPU.  Launches are checked (shape, pointers) and recorded, never run; device pointers are never
// dereferenced.  The product library is never built from this file.
#include <cstdlib>
#include <cstring>
#include <memory>
#include <string>

#include "fs_internal.hpp"

namespace fs {

namespace {
const char* const kNames[K_COUNT] = {"unary", "binary", "reduce_row", "reduce_mid", "transpose_rows", "transpose_tile", "copy",
                                     "softmax_wave", "softmax_block", "layernorm_wave", "layernorm_block", "bias_gelu",
                                     "bias_gelu_dbias", "colfold", "tchain_wave", "tchain_lds", "row_wave", "row_block",
                                     "row_program", "layernorm_bwd", "row_generated"};
long g_launches = 0;

// what any launch must satisfy whatever the kernel: returns a hipError-like code (1 = invalid value)
int check_shape(const LaunchShape& s) {
  const uint64_t threads = (uint64_t)s.block[0] * s.block[1] * s.block[2];
  const uint64_t groups = (uint64_t)s.grid[0] * s.grid[1] * s.grid[2];
  if (threads == 0 || threads > 1024 || groups == 0 || groups > 0x7fffffffull) return 1;
  if (s.lds_bytes > 160u * 1024u) return 1;
  return 0;
}
}  // namespace

int launch_kernel(int32_t kernel, const KernelArgs& args, const LaunchShape& shape, void*) {
  if (kernel < 0 || kernel >= K_COUNT || kernel == K_ROW_GENERATED) return 1;
  if (check_shape(shape)) return 1;
  if (!args.p[0] && kernel != K_ROW_PROGRAM) return 1;   // every compiled-in kernel reads its first pointer
  ++g_launches;
  return 0;
}
int launch_pack(const PackTable& table, void*) {
  if (table.n <= 0 || table.n > kPackMaxMembers || table.total_blocks == 0) return 1;
  for (int i = 0; i < table.n; ++i)
    if (!table.e[i].in[0] || !table.e[i].out) return 1;
  ++g_launches;
  return 0;
}
int launch_fold_many(const FoldManyP& table, uint32_t n_blocks, void*) {
  if (n_blocks == 0) return 0;
  if (table.first_block[0] != 0 || !table.partials[0] || !table.out0[0]) return 1;
  ++g_launches;
  return 0;
}
KernelResources kernel_resources(int32_t, const KernelArgs&) { return KernelResources(); }
KernelResources pack_kernel_resources() { return KernelResources(); }
const char* kernel_name(int32_t k) { return (k >= 0 && k < K_COUNT) ? kNames[k] : "?"; }
const char* hip_error_text(int) { return "launch refused by the host stub"; }

// "compilation" of generated kernels: succeeds when FS_STUB_COMPILE_OK is set (the source is kept, so that identical
// sources share a kernel as in the product), otherwise fails like a missing run-time compiler would
struct GenKernel { std::string source; };
bool gen_available() { return true; }
int gen_compile(const std::string& src, const char* entry, std::shared_ptr<GenKernel>* out, std::string* log) {
  if (getenv("FS_STUB_COMPILE_OK") && entry && src.find(entry) != std::string::npos) {
    *out = std::make_shared<GenKernel>();
    (*out)->source = src;
    return 0;
  }
  if (log) *log = "host stub: no compiler (" + std::to_string(src.size()) + " bytes of source)";
  return 1;
}
GenResources gen_resources(const GenKernel*) { return GenResources(); }
int gen_preload(GenKernel*) { return 0; }
int gen_launch(GenKernel* k, const void* args, size_t args_bytes, const LaunchShape& shape, void*) {
  if (!k || !args || args_bytes == 0 || args_bytes % sizeof(void*) != 0 || check_shape(shape)) return 1;
  ++g_launches;
  return 0;
}

}  // namespace fs

// the entry points that live in .hip files in the product
extern "C" fs_status fs_execute_static(const fs_plan* p, const void* const* inputs, void* const* outputs, void* hip_stream) {
  fs::clear_error();
  const fs_status s = fs::check_execute_args(p, inputs, outputs, "fs_execute_static");
  if (s != FS_OK) return s;
  const fs::Candidate& c = p->candidates[p->chosen];
  if (c.info.workspace_bytes > (int64_t)FS_STATIC_SCRATCH_BYTES)
    return fs::fail(FS_ERR_WORKSPACE, "fs_execute_static: the plan needs %lld bytes of scratch, the static array holds %lld",
                    (long long)c.info.workspace_bytes, (long long)FS_STATIC_SCRATCH_BYTES);
  return fs::run_launches(p, inputs, outputs, reinterpret_cast<void*>(0x7000000), hip_stream, c.launches.size());
}
extern "C" fs_status fs_stream_probe(void*, const void*, size_t, size_t, int32_t, int32_t, int32_t, void*) {
  return fs::fail(FS_ERR_HIP, "fs_stream_probe: not part of the host stub");
}
extern "C" long fs_stub_launch_count(void) { return fs::g_launches; }
