// Internal host-side structures shared by the graph, matcher, cost model and executor.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/fusion_stitching.h"
#include "fs_cost.hpp"
#include "kernels/launch.hpp"

namespace fs {

struct Tensor {
  int32_t dtype = FS_F32;
  int32_t rank = 0;
  int64_t dims[FS_MAX_RANK] = {1, 1, 1, 1};
  int32_t producer = -1;      // op index, -1 for a graph input
  int32_t input_slot = -1;    // position in fs_execute's inputs, -1 if not an input
  int32_t output_slot = -1;   // position in fs_execute's outputs, -1 if not an output
  int32_t store_as = FS_F32;  // storage dtype when it is an output
  std::vector<int32_t> consumers;
  int64_t numel() const {
    int64_t n = 1;
    for (int i = 0; i < rank; ++i) n *= dims[i];
    return n;
  }
};

struct Op {
  int32_t opcode = 0;
  int32_t n_in = 0;
  int32_t in[2] = {-1, -1};
  int32_t out = -1;
  double scalar = 0.0;                     // FS_SCALE / FS_ADD_SCALAR
  int32_t axis = 0;                        // reductions
  int32_t perm[FS_MAX_RANK] = {0, 1, 2, 3};
  int32_t to_dtype = FS_F32;               // FS_CONVERT
};

int dtype_bytes(int32_t dt);
const char* dtype_name(int32_t dt);
const char* opcode_name(int32_t op);
const char* scheme_name(int32_t s);

// status + thread-local message
fs_status fail(fs_status code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();
// the current exception (call inside a catch block) turned into FS_ERR_HOST with a message
fs_status fail_caught(const char* who);

}  // namespace fs

struct fs_graph {
  std::vector<fs::Tensor> tensors;
  std::vector<fs::Op> ops;
  std::vector<int32_t> inputs;   // tensor ids in declaration order
  std::vector<int32_t> outputs;  // tensor ids in declaration order
  // (from, input): graph input `input` is computed outside the graph (say, by a matrix product) from the graph output
  // `from`.  Whatever reads `input` runs after `from` is complete, and never in the kernel that makes `from`.
  std::vector<std::pair<int32_t, int32_t>> external;
  bool finalized = false;
  // per op: the ops whose results it waits for through external computations (sorted, distinct)
  std::vector<std::vector<int>> external_producers() const;
};

namespace fs {

// ---- plan ------------------------------------------------------------------

// One kernel launch of a plan.  `args` is a POD blob the launcher understands;
// pointer fields inside it are filled at execute time from `bind`.
enum BufKind : int32_t { BUF_NONE = 0, BUF_INPUT = 1, BUF_OUTPUT = 2, BUF_WORKSPACE = 3 };
struct BufRef {
  int32_t kind = BUF_NONE;
  int32_t slot = 0;     // input/output slot
  int64_t offset = 0;   // byte offset (workspace)
};

struct Launch {
  int32_t kernel = 0;            // KernelId
  KernelArgs args;               // shapes, flags; pointers patched per execute
  BufRef ptr[kMaxPtrs];          // which buffer each pointer slot takes
  LaunchShape shape;
  std::shared_ptr<GenKernel> gen;   // K_ROW_GENERATED: the compiled kernel, once the plan that chose it is complete
};

// Form in which a matched pattern can join a packed launch (one kernel over many
// independent patterns): one of the row-skeleton specs plus where its operands come from.
struct PackForm {
  int32_t spec = -1;              // PackSpec; -1: this pattern has no packed form
  int32_t in_dt = 0, out_dt = 0;
  uint32_t rows = 0, cols = 0;
  float f[4] = {0, 0, 0, 0};
  int32_t in_slot[2] = {-1, -1};      // fs_execute input slots of the row operands
  int32_t vec_slot[3] = {-1, -1, -1}; // fs_execute input slots of the column vectors
};

struct Candidate {
  fs_plan_info info;
  std::vector<Launch> launches;
  KernelCost cost;               // description of the (single) stitched kernel; unused for unfused plans
  bool fallback = false;         // offered only for the case that no other candidate can be used (the interpreted row
                                 // program beside the kernels generated for the same pattern): passed over by the choice
                                 // while another candidate stands, still reachable by index
};

}  // namespace fs

namespace fs {
// A plan's pattern as a row program with a launch shape: the form in which it can join a generated packed kernel.
struct GenericForm {
  bool valid = false;
  RowProgP prog;
  BufRef ptr[kMaxPtrs];
  uint32_t blocks = 0;
};
}  // namespace fs

struct fs_plan {
  fs::GenericForm generic;
  std::vector<fs::Candidate> candidates;
  int32_t chosen = 0;
  int32_t n_inputs = 0, n_outputs = 0;
  std::vector<int64_t> input_bytes, output_bytes;
  fs::PackForm pack;
  int64_t bytes_min = 0;
  fs_plan_opts opts = {-1, 0, 0, 0};   // what the caller asked for (a re-choice after a failed compile honours it)
};

// Several independent plans that run as one packed launch per 32 members.
struct fs_pack {
  struct Member {
    fs::PackForm form;
    int32_t first_input = 0, n_inputs = 0, first_output = 0;
  };
  std::vector<Member> members;
  std::vector<fs::PackTable> tables;   // one per launch, pointers left null
  // generated form: one kernel per launch, made for exactly these members
  struct PtrRef { int32_t kind; int32_t index; };   // BUF_INPUT / BUF_OUTPUT, position in fs_pack_execute's arrays
  struct GenLaunch {
    std::shared_ptr<fs::GenKernel> kernel;
    uint32_t blocks = 0;
    std::vector<PtrRef> ptrs;
  };
  std::vector<GenLaunch> generated;    // non-empty: these run instead of `tables`
  fs_pack_info info{};
  int32_t n_inputs = 0, n_outputs = 0;
};

namespace fs {

// matcher + candidate enumeration (fs_match.cpp / fs_cost.cpp)
fs_status build_unfused(const fs_graph& g, Candidate* out);
// Appends every stitched candidate that fits `g`; returns the pattern name or "" if none matches.
// `pack` (may be null) receives the pattern's packed form when it has one.
std::string build_stitched(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
// Candidates that run `g` as an interpreted row program (fs_rowprog.cpp); false if `g` is not a
// pattern of element-wise ops and last-axis reductions over one row space.
bool build_row_program(const fs_graph& g, std::vector<Candidate>* out);
// Generated row kernels (fs_codegen.cpp): HIP source of the kernel specialised to the program `p` and its
// launch shape; the body alone (without the embedded device headers) for listings.
std::string generate_row_kernel(const RowProgP& p);
std::string generate_row_kernel_body(const RowProgP& p);
std::string generated_kernel_entry(const RowProgP& p);   // fs_gen_row_<hash of the source>
// Source (without the embedded device headers, see embedded_prelude) of one kernel that runs several row programs,
// member m on workgroups [sum of blocks before m, + blocks[m]); ptr_slots[m]: the members' pointer slots in the
// order of the kernel's pointer table; *entry: the kernel's name.
std::string generate_pack_kernel(const std::vector<RowProgP>& members, const std::vector<uint32_t>& blocks,
                                 std::vector<std::vector<int>>* ptr_slots, std::string* entry);
std::string embedded_prelude();
// Pairs of row reductions "rmax; acc - max; exp; rsum" that a row worked through in chunks gathers in one pass
// (online[q] = 1 for the first of each pair; `online` may be null); returns their number.
int online_reduction_pairs(const RowProgP& p, std::vector<char>* online);
// Process-wide switch: candidates with generated kernels are offered only while it is on (default: on
// unless the environment says FS_CODEGEN=0) and the run-time compiler is available.
bool codegen_enabled();
// fs_plan_create without the last step: generated kernels are not compiled yet.  complete_plan() compiles
// the chosen candidate's kernel; if that fails, or the kernel spills registers, it moves the choice to the
// next best candidate (unless the caller fixed the candidate, then it fails).
fs_status create_plan(const fs_graph* g, int32_t scheme, const fs_plan_opts* opts, bool complete, fs_plan** out);
// The first `n_launches` launches of the plan's chosen candidate (arguments already validated by the caller).
fs_status run_launches(const fs_plan* p, const void* const* inputs, void* const* outputs, void* workspace, void* hip_stream,
                       size_t n_launches);
// The checks every execute entry point makes on its pointer arrays (null, alignment); `who` names the caller in the message.
fs_status check_execute_args(const fs_plan* p, const void* const* inputs, void* const* outputs, const char* who);
// How many kernel launches that makes (folds of column partial sums that follow each other go out as one).
size_t launches_issued(const fs_plan* p, size_t n_launches);
fs_status complete_plan(fs_plan* p);
int64_t graph_bytes_min(const fs_graph& g);
// Multiply-high constants for n / d with n < 2^31 (d == 0 in the result marks "no usable constants").
FastDiv make_fastdiv(uint32_t d);
void predict(Candidate* c);  // fills info.predicted_us, waves_per_simd, vgprs, lds

}  // namespace fs
