/*
 * fusion_stitching.h -- C ABI of the MI355X (gfx950) stitched-subgraph library.
 *
 * The library executes one *fusion pattern* -- a subgraph of memory-intensive
 * ops (element-wise, broadcast, reduction, transpose; the op kinds of paper
 * Section 1 and Section 3.1; Section 5.1, "fusion pattern P_i = (V_i, E_i)") --
 * either as one stitched GPU kernel in which intermediates stay on chip, or as
 * the per-op baseline of one kernel per op.  The calls mirror the paper's
 * code-generation problem statement (Section 4: a fusion pattern goes in, a
 * kernel with a chosen schedule and launch dimension comes out, Section 4.2).
 * The kernel is a hand-written one of a pattern family where a family matches
 * the pattern, otherwise HIP source generated for the pattern and compiled for
 * gfx950 when the plan is created (or, without the run-time compiler, a fixed
 * kernel that interprets the pattern's instruction list).
 *
 * Conventions
 *   - All handles are opaque and owned by the library; destroy with the
 *     matching *_destroy.  Every pointer passed to fs_execute / fs_stream_copy
 *     is DEVICE memory owned by the caller; every other pointer is HOST memory.
 *   - No call throws or aborts.  Calls returning fs_status give FS_OK (0) or a
 *     negative error; calls returning fs_tensor give an id >= 0 or a negative
 *     error.  fs_last_error() gives the text of the calling thread's last error.
 *   - Tensors are dense, row-major, rank 1..FS_MAX_RANK, fewer than 2^31 elements.
 *   - Arithmetic is float32 whatever the storage dtype; conversion to a
 *     16-bit storage dtype rounds to nearest-even at the final store.
 */
#ifndef FUSION_STITCHING_H
#define FUSION_STITCHING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FS_MAX_RANK 4

typedef struct fs_graph fs_graph;
typedef struct fs_plan fs_plan;
typedef struct fs_pack fs_pack;
typedef struct fs_program fs_program;
typedef int32_t fs_status;
typedef int32_t fs_tensor;

enum fs_error {
  FS_OK = 0,
  FS_ERR_INVALID_ARG = -1,         /* null pointer, bad enum value, bad id, graph not finalized, ...  */
  FS_ERR_SHAPE = -2,               /* operand shapes do not broadcast / bad axis / bad perm / too large */
  FS_ERR_DTYPE = -3,               /* dtype not accepted by the op                                    */
  FS_ERR_CYCLE = -4,               /* an operand id does not precede the op (graphs are built in
                                      topological order, so a cycle can only show up this way;
                                      Section 5.2 discards cyclic patterns)                            */
  FS_ERR_UNSUPPORTED_PATTERN = -5, /* a stitched scheme was asked for and no stitched kernel matches
                                      (Section 5.2: only patterns the code generator can process)      */
  FS_ERR_LOCALITY = -6,            /* forced scheme / shape breaks the reuse-scope locality rule
                                      (Section 4.2: schedules violating data locality are discarded)   */
  FS_ERR_WORKSPACE = -7,           /* workspace null or smaller than fs_plan_info.workspace_bytes      */
  FS_ERR_ALIGN = -8,               /* a device pointer is not 16-byte aligned                          */
  FS_ERR_HIP = -9,                 /* a HIP call failed; text carries hipGetErrorString                */
  FS_ERR_HOST = -10                /* the host ran out of memory, or an internal error was caught at the
                                      boundary (nothing is ever thrown across it)                       */
};

enum fs_dtype { FS_F32 = 0, FS_F16 = 1, FS_BF16 = 2, FS_I32 = 3 };

/* Memory-intensive op vocabulary (Section 4: light element-wise, expensive
 * element-wise, reduction; Section 3.1: broadcast; plus transpose and convert).
 * Binary ops broadcast numpy-style (ranks right-aligned, extent 1 stretches).
 * Reductions keep the reduced axis with extent 1.  Results are FS_F32 except
 * FS_TRANSPOSE (keeps its operand's dtype, moves raw bits) and FS_CONVERT.     */
enum fs_opcode {
  FS_ADD = 0, FS_SUB = 1, FS_MUL = 2, FS_DIV = 3, FS_MAX = 4, /* 2 operands, attr: none            */
  FS_SCALE = 5,          /* x * value                      attr: fs_attr_scalar                    */
  FS_ADD_SCALAR = 6,     /* x + value                      attr: fs_attr_scalar                    */
  FS_SQUARE = 7, FS_EXP = 8, FS_RSQRT = 9, FS_TANH = 10,      /* 1 operand, attr: none             */
  FS_GELU_TANH = 11,     /* z/2 (1 + tanh(sqrt(2/pi)(z + 0.044715 z^3)))                           */
  FS_GELU_TANH_GRAD = 12,/* d/dz of FS_GELU_TANH                                                   */
  FS_BROADCAST = 13,     /* stretch to attr dims           attr: fs_attr_dims                      */
  FS_REDUCE_SUM = 14, FS_REDUCE_MAX = 15, FS_REDUCE_MEAN = 16, /* attr: fs_attr_axis               */
  FS_TRANSPOSE = 17,     /* out.dims[i] = in.dims[perm[i]] attr: fs_attr_perm                      */
  FS_CONVERT = 18,       /* round to dtype                 attr: fs_attr_dtype                     */
  FS_LOG = 19,           /* natural logarithm                                                      */
  FS_SIGMOID = 20,       /* 1 / (1 + exp(-x))                                                      */
  FS_RELU = 21,          /* max(x, 0)                                                              */
  FS_ABS = 22, FS_SQRT = 23,                                  /* 1 operand, attr: none             */
  FS_OPCODE_COUNT = 24
};

typedef struct fs_attr_scalar { double value; } fs_attr_scalar;
typedef struct fs_attr_axis { int32_t axis; } fs_attr_axis;               /* 0 <= axis < rank        */
typedef struct fs_attr_perm { int32_t perm[FS_MAX_RANK]; } fs_attr_perm;   /* first `rank` entries    */
typedef struct fs_attr_dims { int32_t rank; int64_t dims[FS_MAX_RANK]; } fs_attr_dims;
typedef struct fs_attr_dtype { int32_t dtype; } fs_attr_dtype;

/* Composition schemes (Section 4.1).  LOCAL = kernel packing + thread composition
 * (values stay in the lane that made them); WAVE = warp composition on a 64-wide
 * wavefront (cross-lane DPP / permute); LDS = block composition (reduced values
 * and tiles go through LDS); GLOBAL = one hand-off through device memory between
 * workgroups, which the paper leaves out (Section 4.1, last paragraph) and which
 * the column-reduction pattern needs; UNFUSED = one kernel per op; AUTO = the
 * cost model chooses among the stitched candidates and falls back to UNFUSED
 * when no stitched kernel matches.                                              */
enum fs_scheme {
  FS_SCHEME_AUTO = 0, FS_SCHEME_UNFUSED = 1, FS_SCHEME_LOCAL = 2,
  FS_SCHEME_WAVE = 3, FS_SCHEME_LDS = 4, FS_SCHEME_GLOBAL = 5
};

/* Optional constraints on the launch shape; a zero / negative field means "any", so a
 * zero-initialised struct asks for nothing.  The cost model picks the cheapest candidate
 * that satisfies all given fields; if none does, fs_plan_create returns FS_ERR_LOCALITY.
 * `candidate` overrides the choice: with k > 0 the plan is entry k - 1 of the candidate
 * list, whatever the model and the other fields say.                                  */
typedef struct fs_plan_opts {
  int32_t candidate;      /* k > 0: take exactly entry k - 1 of the candidate list (the index
                             fs_plan_info.candidate reports, plus one); <= 0: choose           */
  int32_t block_threads;  /* threads per workgroup                                             */
  int32_t lanes_per_row;  /* lanes that share one reduction row (WAVE) / threads per row (LDS) */
  int32_t vecs_per_lane;  /* 128-bit vectors each lane keeps in registers                      */
} fs_plan_opts;

/* What a plan will do (Section 4.3: latency is estimated from launch dimension,
 * shared-memory use and register use; here registers and LDS are the compiled
 * kernel's own figures).                                                         */
typedef struct fs_plan_info {
  int32_t scheme;            /* enum fs_scheme actually used                                   */
  int32_t n_kernels;         /* launches per fs_execute                                        */
  int32_t block[3];          /* workgroup shape of the dominant kernel                         */
  int32_t grid[3];           /* workgroups of the dominant kernel                              */
  int32_t lanes_per_row;
  int32_t vecs_per_lane;
  int32_t rows_per_block;
  int32_t lds_bytes;         /* LDS per workgroup                                              */
  int32_t vgprs;             /* vector registers per lane (compiled figure, or an estimate
                                when no device is present)                                     */
  int32_t waves_per_simd;    /* occupancy the model derived from vgprs / lds / block shape     */
  int32_t n_candidates;      /* size of the enumerated candidate list                          */
  int32_t candidate;         /* index of the chosen one                                        */
  int64_t workspace_bytes;   /* device scratch fs_execute needs (may be 0)                     */
  int64_t bytes_min;         /* each subgraph input read once + each output written once       */
  int64_t bytes_moved_model; /* bytes the plan's kernels move according to the model           */
  double predicted_us;       /* cost-model estimate for one fs_execute                         */
  char pattern[32];          /* matched stitched pattern, or "unfused"                         */
  char kernel[64];           /* name of the dominant kernel variant                            */
} fs_plan_info;

/* ---- graph descriptor (Section 5.1: a fusion pattern is a subgraph) ---------- */

/* New empty graph.  *out receives the handle.  Errors: FS_ERR_INVALID_ARG.      */
fs_status fs_graph_create(fs_graph **out);
/* Frees the graph (null is accepted).  Plans made from it stay valid.           */
void fs_graph_destroy(fs_graph *g);
/* Declares a subgraph input of `rank` extents dims[0..rank) (host array, copied).
 * fs_execute's `inputs` follow the order of these calls.
 * Errors: FS_ERR_INVALID_ARG (null, bad dtype, finalized graph), FS_ERR_SHAPE.   */
fs_tensor fs_graph_input(fs_graph *g, int32_t dtype, int32_t rank, const int64_t *dims);
/* Appends op `opcode` over operands in[0..n_in) (host array of earlier ids) with
 * the attribute struct named beside the opcode (host, copied; null when the op
 * has none).  Returns the id of its result tensor.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_CYCLE, FS_ERR_SHAPE, FS_ERR_DTYPE.          */
fs_tensor fs_graph_op(fs_graph *g, int32_t opcode, int32_t n_in, const fs_tensor *in,
                      const void *attr, size_t attr_bytes);
/* Marks tensor t as a subgraph output stored as `store_as`.  fs_execute's
 * `outputs` follow the order of these calls.  A tensor can be marked once.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_DTYPE (I32 tensors only store as I32).      */
fs_status fs_graph_output(fs_graph *g, fs_tensor t, int32_t store_as);
/* Declares that graph input `input` is computed OUTSIDE the graph (by a matrix product,
 * say) from the op result `from`, which must be declared a graph output before
 * fs_graph_finalize.  Section 1 / Section 5.1: compute-intensive ops are not fused; they cut the graph
 * of memory-intensive ops, and this call records the cut.  Consequences: no fusion pattern
 * holds both the op that makes `from` and an op that reads `input` (nor ops on a path
 * between two of its members that leads through such a dependence); the steps of an explored
 * program are grouped into stages (fs_program_execute_stage) between which the caller runs
 * the external computations.  Call it after the op that makes `from` and before any op
 * reads `input`.  A graph with such dependences has no single plan: fs_plan_create returns
 * FS_ERR_UNSUPPORTED_PATTERN; use fs_explore.  Errors: FS_ERR_INVALID_ARG.                */
fs_status fs_graph_external(fs_graph *g, fs_tensor from, fs_tensor input);
/* Freezes the graph: at least one output, every op reaches an output.
 * Errors: FS_ERR_INVALID_ARG.                                                    */
fs_status fs_graph_finalize(fs_graph *g);

/* ---- plan (Section 4.2: enumerate schedules and launch dimensions, discard
 *      those that break locality, keep the cheapest by the evaluator) ----------- */

/* Builds a plan for a finalized graph.  `opts` may be null.  *out receives the
 * handle.  Needs no GPU (register figures fall back to estimates without one).
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_UNSUPPORTED_PATTERN, FS_ERR_LOCALITY.        */
fs_status fs_plan_create(const fs_graph *g, int32_t scheme, const fs_plan_opts *opts, fs_plan **out);
void fs_plan_destroy(fs_plan *p);
/* Fills *out (host) with the chosen candidate's figures.                         */
fs_status fs_plan_query(const fs_plan *p, fs_plan_info *out);
/* Fills *out with the figures of entry `index` (0 <= index < n_candidates) of the
 * list the plan was chosen from, in enumeration order.                           */
fs_status fs_plan_candidate(const fs_plan *p, int32_t index, fs_plan_info *out);

/* Writes a text listing of what the plan will run into `text` (HOST buffer of `capacity`
 * bytes, always NUL-terminated when capacity > 0; truncated if too small) and returns
 * the size needed for the whole listing including the NUL, or a negative error.  One
 * line per launch (kernel, grid, block, dynamic LDS) and per buffer binding (a generated
 * kernel also `entry <name of its entry point>`, the name kernel traces show); for a
 * pattern that runs as a row program (the generic path for patterns no hand-written
 * kernel covers, Section 4.2; interpreted or as a generated kernel) also its register
 * files, the extents of the leading axes (`lead=a,b,c`), for operands and outputs that
 * are stretched or transposed along them their row strides (`rowstrides=m0,m1,m2`: row
 * (c0,c1,c2) of the pattern is row c0*m0+c1*m1+c2*m2 of that buffer), and one line per
 * instruction of its accumulator machine: `instr <n> <op> b=<kind>:<index> dst=<index>
 * flags=<v|s><k|-> aux=<dtype> imm=<value>` (v: acc <- acc op b on full-shaped values,
 * s: the same on per-row values; k: result also kept in register dst).  A pattern with
 * sums over all rows adds `colsums <n> partials <buffer> rows_per_group <r> col_tiles <t>`
 * (and `launch colfold` entries after it, one per fold; folds that follow each other
 * are issued as ONE kernel launch, which `launches=` counts); a row worked through in pieces adds
 * `chunks <n> of <w> columns[, the first <k> kept in registers]`.
 * Errors: FS_ERR_INVALID_ARG.                                                          */
int64_t fs_plan_describe(const fs_plan *p, char *text, size_t capacity);

/* ---- generated kernels (Section 4: the code generator turns a fusion pattern into one
 * kernel) -------------------------------------------------------------------------
 * A pattern that no hand-written kernel family covers, but whose reuse stays inside a
 * row, is offered in two forms: as an interpreted row program (one fixed kernel walks an
 * instruction list) and as a generated kernel (HIP source specialised to the pattern, its
 * extents and its launch shape, compiled for gfx950 by the HIP run-time compiler when the
 * plan is created; fs_plan_info.kernel then starts with "row_generated").  Compiled kernels
 * are shared between plans with identical source and stay loaded until the process ends.
 * Generated kernels only: row lengths that are no multiple of 4 elements; rows of more than
 * 2048 128-bit vectors (workgroups of 512 / 1024 threads; beyond 8192 vectors the row is
 * worked through in chunks, one pass per row reduction, the chunks kept in registers where
 * they fit); sums over all rows of a pattern (reduce_sum along axis 0 of a rank-2 value, or
 * a chain of reduce_sums along each leading axis in turn; a graph output nothing else
 * reads, float32 or rounded once to a 16-bit dtype; the plan then has a workspace and a
 * second launch that folds the partial sums); more than 4 full-shaped inputs.
 * Compilation needs no GPU; the module is loaded on the device that is current at plan
 * creation (or, without one, by the first fs_execute: do that one outside stream capture).
 * If the compiler is not available, compilation fails or the kernel would spill registers,
 * the choice falls back to the next best candidate (for FS_SCHEME_AUTO in the end to the
 * per-op plan).  Environment: FS_CODEGEN=0 switches generated kernels off by default;
 * FS_CODEGEN_CACHE_DIR=<existing directory> keeps compiled code objects there between
 * processes (files fs_gfx950_<hash>.co, verified against the full source when read).    */

/* Process-wide switch for offering generated kernels (default 1; the environment variable
 * FS_CODEGEN=0 sets the default to 0).  Affects plans, scores and programs created
 * afterwards.  Returns the previous effective setting.                                 */
int32_t fs_codegen_enable(int32_t on);
/* 1 if the run-time compiler could be loaded in this process, else 0.                 */
int32_t fs_codegen_available(void);
/* Writes the HIP source of the plan's generated kernel(s) (the kernel function only, not
 * the fixed device headers it is compiled with) into `text` (HOST buffer of `capacity`
 * bytes, NUL-terminated, truncated if too small) and returns the size needed including
 * the NUL (1 for a plan without a generated kernel), or a negative error.
 * Errors: FS_ERR_INVALID_ARG.                                                          */
int64_t fs_plan_source(const fs_plan *p, char *text, size_t capacity);

/* ---- execution (the run-time hot path) --------------------------------------- */

/* Enqueues the plan's kernel(s) on `hip_stream` (a hipStream_t; null = the
 * default stream) and returns without waiting.  inputs[i] / outputs[j] are
 * DEVICE pointers in declaration order, each 16-byte aligned and sized for its
 * tensor; inputs are never written.  `workspace` is DEVICE scratch of at least
 * fs_plan_info.workspace_bytes (may be null when that is 0); its contents on entry
 * do not matter (every kernel that reads it reads what an earlier kernel of the same
 * call wrote) and it is reusable afterwards.  Allocates nothing, never
 * synchronizes.  Two calls that share a workspace must be ordered on one stream.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_WORKSPACE, FS_ERR_ALIGN, FS_ERR_HIP.         */
fs_status fs_execute(const fs_plan *p, const void *const *inputs, void *const *outputs,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* fs_execute for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and rules, without
 * the workspace: the plan's scratch (the partial column sums that the workgroups of one
 * launch hand to the fold launch, or a per-op plan's intermediates) is a fixed array of
 * FS_STATIC_SCRATCH_BYTES in the library's device image, one copy per GPU, held until the
 * process ends; the device of `hip_stream` must be the current device.  A plan whose
 * fs_plan_info.workspace_bytes is larger is refused with FS_ERR_WORKSPACE before anything
 * is enqueued.  Allocates nothing on the device (no hipMalloc / hipFree, no allocating
 * library call), never synchronizes; the first call on a GPU looks up the array's address.
 * Every call on a GPU uses that GPU's one array, so two calls whose kernels may overlap in
 * time (different streams, or graphs replayed concurrently) race: order them on one stream.
 * The array keeps the last call's contents; no plan needs it cleared.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_WORKSPACE, FS_ERR_ALIGN, FS_ERR_HIP.               */
#define FS_STATIC_SCRATCH_BYTES (4u << 20)
fs_status fs_execute_static(const fs_plan *p, const void *const *inputs, void *const *outputs, void *hip_stream);

/* ---- packed execution (Section 4.1, kernel packing: ops with no data dependence
 *      share one kernel to cut launches; Section 5.2, remote fusion: patterns that
 *      are not adjacent in the graph may still be packed) -------------------------- */

#define FS_PACK_MAX_MEMBERS 256  /* members of one pack; every 32 of them share one launch */

typedef struct fs_pack_info {
  int32_t n_members;
  int32_t n_kernels;            /* launches per fs_pack_execute = ceil(n_members / 32)          */
  int32_t grid, block;          /* workgroups over all launches, threads per workgroup          */
  int32_t vgprs;                /* registers per lane of the packed kernel (0 without a device) */
  int32_t n_inputs, n_outputs;  /* lengths of fs_pack_execute's pointer arrays                  */
  int32_t generated;            /* 1: the pack runs kernels generated for exactly its members   */
  int64_t bytes_min;            /* sum of the members' bytes_min                                */
  double predicted_us;          /* model estimate for one fs_pack_execute                       */
  double predicted_separate_us; /* sum of the members' own predicted_us (one launch each)       */
} fs_pack_info;

/* Packs plans[0..n) -- independent patterns, none reading another's output -- into
 * one object whose execution runs all of them in ceil(n/32) launches.  Two forms:
 *   generated (where the run-time compiler is available, see fs_codegen_enable): every
 *     member is any plan, not made with FS_SCHEME_UNFUSED, whose pattern is row-local
 *     (what runs as a row program: element-wise ops, broadcasts, last-axis reductions,
 *     transposes of leading axes; no column sums); one kernel per launch is generated
 *     with a device function per member;
 *   fixed (otherwise): one pre-compiled kernel reads a table of members; a member's
 *     pattern must be softmax without mask, softmax backward, RMS norm, LayerNorm with
 *     affine output (alone, or with residual and bias) or bias + GELU; input and output
 *     storage of the same dtype (LayerNorm also float32 -> bfloat16); rows of at most
 *     1024 128-bit vectors.
 * The plans may be destroyed afterwards; the pack keeps what it needs.  `plans` is a
 * HOST array.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_UNSUPPORTED_PATTERN (names the member),
 * FS_ERR_LOCALITY (a member's row is too long for one workgroup), FS_ERR_SHAPE.      */
fs_status fs_pack_create(const fs_plan *const *plans, int32_t n, fs_pack **out);
void fs_pack_destroy(fs_pack *p);
fs_status fs_pack_query(const fs_pack *p, fs_pack_info *out);
/* Enqueues the packed launch(es) on `hip_stream` and returns without waiting.
 * `inputs` holds the members' inputs one member after the other (member 0's inputs in
 * its graph's declaration order, then member 1's, ...), `outputs` likewise; HOST arrays
 * of DEVICE pointers, each 16-byte aligned.  Members must not alias each other's
 * outputs.  Needs no workspace, allocates nothing, never synchronizes.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_ALIGN, FS_ERR_HIP.                              */
fs_status fs_pack_execute(const fs_pack *p, const void *const *inputs, void *const *outputs, void *hip_stream);

/* ---- fusion exploration over a multi-pattern graph (Section 5) ------------------- */

/* Zero fields take the paper's settings: the 3 best candidate patterns per vertex
 * (Section 5.2), beam width 3 (Section 5.3), packing of launch-bound patterns on.     */
typedef struct fs_explore_opts {
  int32_t top_k;        /* candidate patterns kept per vertex and per consumer group, 1..16 */
  int32_t beam_width;   /* candidate fusion plans kept while traversing the graph, 1..16    */
  int32_t no_packing;   /* 1: leave independent launch-bound patterns in launches of their own */
  int32_t no_remote_fusion; /* 1: do not merge patterns that no edge joins (Section 5.2, remote fusion) */
  int32_t no_joint_folds;   /* 1: every pattern with column sums finishes them in launches of its own     */
} fs_explore_opts;

typedef struct fs_program_info {
  int32_t n_ops;          /* ops of the graph                                             */
  int32_t n_patterns;     /* fusion patterns of two or more ops in the chosen plan         */
  int32_t n_single_ops;   /* ops left in a kernel of their own                             */
  int32_t n_steps;        /* fs_execute / packed launches issued per fs_program_execute    */
  int32_t n_kernels;      /* kernel launches per fs_program_execute                        */
  int32_t n_packs;        /* packed launches among the steps                               */
  int32_t beam_plans;     /* candidate plans the final choice was made among               */
  int32_t n_joint_folds;  /* column-sum folds moved behind the last step and issued as one launch (per 8): sums over
                             all rows that nothing in the graph reads need only be complete when the program ends */
  int64_t workspace_bytes;   /* device scratch fs_program_execute needs                    */
  int64_t bytes_min;         /* graph inputs read once + graph outputs written once        */
  int64_t bytes_moved_model; /* bytes the plan's kernels move, tensors between patterns included */
  double f_total_us;         /* sum of the chosen patterns' delta-evaluator scores (Eq. 3), remote fusion included */
  double predicted_us;       /* latency-evaluator estimate of one fs_program_execute        */
  double predicted_unfused_us; /* the same ops one kernel each, by the delta-evaluator's per-op term */
  int32_t n_stages;       /* 1 + the longest chain of external computations (fs_graph_external) between steps */
  int32_t reserved;
} fs_program_info;

/* Delta-evaluator (Section 5.4, Eq. 3) for the ops[0..n) of `g` (op index = order of the
 * fs_graph_op calls) taken as ONE fusion pattern: *f_us receives
 * T_reduced_mem + T_reduced_calls - T_penalty in microseconds (0 for a single op).
 * *f_optimistic_us (may be null) receives the score the pattern would have if one kernel
 * ran it at streaming rate; it is set whenever the ops form a pattern without a cyclic
 * dependence, also when the call fails with FS_ERR_UNSUPPORTED_PATTERN (the explorer
 * grows such patterns further, in case a larger one is covered by a kernel family).
 * `ops`, `f_us`, `f_optimistic_us` are HOST pointers.  Errors: FS_ERR_INVALID_ARG; FS_ERR_CYCLE (fusing
 * them creates a cyclic dependence, Section 5.2, or they hold both ends of an external
 * computation declared with fs_graph_external); FS_ERR_UNSUPPORTED_PATTERN (no stitched
 * kernel can run them as one pattern); FS_ERR_DTYPE (a graph output stored in another
 * dtype than it was computed in would have to feed ops outside the pattern).            */
fs_status fs_explore_score(const fs_graph *g, const int32_t *ops, int32_t n, double *f_us, double *f_optimistic_us);

/* Searches a fusion plan for a finalized graph that may hold many patterns (Section 5.2:
 * candidate patterns per vertex by PatternReduction in post-order; Section 5.3: beam
 * search over the vertices, final choice by the latency evaluator) and builds the
 * executable program: one plan per chosen pattern, one per op left alone, packed launches
 * for independent launch-bound patterns (remote fusion, Section 5.2).  `opts` may be null.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_DTYPE (see fs_explore_score; add an explicit convert
 * op and let the consumers read its result), FS_ERR_UNSUPPORTED_PATTERN, FS_ERR_SHAPE.  */
fs_status fs_explore(const fs_graph *g, const fs_explore_opts *opts, fs_program **out);
void fs_program_destroy(fs_program *p);
fs_status fs_program_query(const fs_program *p, fs_program_info *out);
/* Step `index` (0 <= index < n_patterns + n_single_ops, in execution order): its op
 * indices in graph order into ops[0..capacity) (HOST; may be null), their number into
 * *n_ops, its delta-evaluator score, the packed launch it belongs to (-1: none) and the
 * figures of its plan.  Every out pointer may be null.  Errors: FS_ERR_INVALID_ARG.      */
fs_status fs_program_pattern(const fs_program *p, int32_t index, int32_t *ops, int32_t capacity, int32_t *n_ops,
                             double *f_us, int32_t *pack, fs_plan_info *info);
/* Writes a text listing of what fs_program_execute will issue into `text` (HOST buffer of
 * `capacity` bytes, NUL-terminated, truncated if too small) and returns the size needed
 * including the NUL, or a negative error.  One line per step in execution order (`step <i>
 * ops=<graph op indices> pattern=<name> kernel=<name> launches=<issued at the step> f_us=<score>`,
 * with `pack=<j>` for members of a packed launch, which is issued where its first member
 * stands, and `stage=<k>` when the program has more than one stage), indented under it where each of the plan's inputs and outputs lives (`in<k>` /
 * `out<k>` of the graph, or `ws+<offset>` in the program's workspace) and the plan's own
 * scratch (`scratch ws+<offset> <bytes>`); then one line per packed launch (`pack <j>
 * launches=<n> members=<steps>`) and per joint fold launch (`joint_fold <j> folds=<n>
 * of_steps=<steps whose column sums it finishes>`).  Errors: FS_ERR_INVALID_ARG.         */
int64_t fs_program_describe(const fs_program *p, char *text, size_t capacity);
/* Enqueues the whole program on `hip_stream` and returns without waiting.  inputs /
 * outputs: DEVICE pointers in the graph's declaration order, 16-byte aligned.  `workspace`:
 * DEVICE scratch of at least fs_program_info.workspace_bytes, 256-byte aligned (it holds the
 * tensors that cross from one pattern to the next and the patterns' own scratch; its contents
 * on entry do not matter); calls that share it must be ordered on one stream.
 * Allocates nothing, never synchronizes.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_WORKSPACE, FS_ERR_ALIGN, FS_ERR_HIP.               */
fs_status fs_program_execute(const fs_program *p, const void *const *inputs, void *const *outputs, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* The steps of one stage (0 <= stage < fs_program_info.n_stages), same arguments and rules.
 * A program whose graph declares external computations (fs_graph_external) is run stage by
 * stage: after stage k the caller runs, on the same stream, the external computations whose
 * operands are complete (every graph output that feeds one is written by the end of the
 * stage that makes it) and whose results stage k+1 reads.  fs_program_execute issues all
 * stages back to back (for timing the program's own kernels with the external results
 * already in place).  Column sums that nothing reads, external computations included, may
 * only be complete after the LAST stage (their joint fold launch runs there).
 * Errors: as fs_program_execute.                                                           */
fs_status fs_program_execute_stage(const fs_program *p, int32_t stage, const void *const *inputs, void *const *outputs,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Plain streaming copy of `bytes` (multiple of 16) from src to dst, both DEVICE
 * and 16-byte aligned: the measured HBM ceiling every result is reported beside
 * (Section 2.2 names off-chip traffic as the dominant cost).                     */
fs_status fs_stream_copy(void *dst, const void *src, size_t bytes, void *hip_stream);

/* Streaming probe: a kernel that only moves data, with a chosen mix of streams, in the
 * one-shot shape of the stitched row kernels.  Every lane reads `vecs_per_lane` (1, 2 or 4)
 * 128-bit vectors from each of `reads` (0..4) input streams and writes as many to each of
 * `writes` (0..2, not both 0) output streams; all loads are issued before the first store.
 * Stream r of a side starts stream_pitch_bytes * r behind the side's pointer (0 = stream_bytes:
 * the streams follow each other; a larger pitch puts a gap between them, for experiments
 * with the streams' relative placement -- none measured so far changed the time).
 * `src`: DEVICE, (reads - 1) * pitch + stream_bytes (may be null when reads is 0); `dst`:
 * DEVICE, likewise for writes, at least 16 bytes (a read-only probe stores nothing there unless
 * the input holds one particular bit pattern, which keeps its loads alive); stream_bytes and
 * the pitch multiples of 16, below 2^35; pointers 16-byte aligned.  What it writes is a function of the
 * inputs and the element index, of no further meaning.  Its time is the reference a stitched
 * kernel with the same bytes and the same read : write mix is reported beside (Section
 * 2.2: traffic is what these ops cost); the read-only and write-only rates on a large
 * size give a bound (read bytes / read rate + written bytes / write rate); with a small
 * stream_bytes it gives the fixed cost of a launch of that many workgroups.
 * Errors: FS_ERR_INVALID_ARG, FS_ERR_ALIGN, FS_ERR_SHAPE, FS_ERR_HIP.                    */
fs_status fs_stream_probe(void *dst, const void *src, size_t stream_bytes, size_t stream_pitch_bytes, int32_t reads,
                          int32_t writes, int32_t vecs_per_lane, void *hip_stream);

/* Text of the calling thread's most recent error ("" if none); valid until the
 * thread's next library call.                                                    */
const char *fs_last_error(void);
/* Library version string (static storage).                                       */
const char *fs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FUSION_STITCHING_H */
