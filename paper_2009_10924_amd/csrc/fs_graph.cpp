// Op-graph descriptor: construction, shape / dtype inference, validation.
// A graph is one fusion pattern (paper Section 5.1): tensors are vertices' results,
// operands are edges.  Ops are appended in topological order, so operand ids must
// be smaller than the id of the result they feed.
#include <cstring>

#include <algorithm>
#include <exception>
#include <new>

#include "fs_internal.hpp"

namespace fs {

// fixed storage: reporting an error must not itself need host memory
static thread_local char g_error[1024];

fs_status fail(fs_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof g_error, fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_error[0] = 0; }

// Called from the catch (...) of every C-ABI function: nothing may be thrown across the boundary.
fs_status fail_caught(const char* who) {
  try {
    throw;
  } catch (const std::bad_alloc&) {
    return fail(FS_ERR_HOST, "%s: out of host memory", who);
  } catch (const std::exception& e) {
    return fail(FS_ERR_HOST, "%s: internal error: %s", who, e.what());
  } catch (...) {
    return fail(FS_ERR_HOST, "%s: internal error", who);
  }
}

int dtype_bytes(int32_t dt) { return (dt == FS_F32 || dt == FS_I32) ? 4 : 2; }
const char* dtype_name(int32_t dt) {
  switch (dt) {
    case FS_F32: return "f32";
    case FS_F16: return "f16";
    case FS_BF16: return "bf16";
    case FS_I32: return "i32";
    default: return "?";
  }
}
const char* opcode_name(int32_t op) {
  static const char* names[FS_OPCODE_COUNT] = {
      "add", "sub", "mul", "div", "max", "scale", "add_scalar", "square", "exp", "rsqrt", "tanh",
      "gelu_tanh", "gelu_tanh_grad", "broadcast", "reduce_sum", "reduce_max", "reduce_mean", "transpose", "convert",
      "log", "sigmoid", "relu", "abs", "sqrt"};
  return (op >= 0 && op < FS_OPCODE_COUNT) ? names[op] : "?";
}
const char* scheme_name(int32_t s) {
  static const char* names[] = {"auto", "unfused", "local", "wave", "lds", "global"};
  return (s >= 0 && s <= FS_SCHEME_GLOBAL) ? names[s] : "?";
}

static bool valid_dtype(int32_t dt) { return dt >= FS_F32 && dt <= FS_I32; }
static bool float_dtype(int32_t dt) { return dt == FS_F32 || dt == FS_F16 || dt == FS_BF16; }

static int operand_count(int32_t opcode) { return opcode <= FS_MAX ? 2 : 1; }

}  // namespace fs

using namespace fs;

extern "C" {

const char* fs_last_error(void) { return g_error; }
const char* fs_version(void) { return "fusion-stitching-gfx950 0.1"; }

fs_status fs_graph_create(fs_graph** out) try {
  clear_error();
  if (!out) return fail(FS_ERR_INVALID_ARG, "fs_graph_create: out is null");
  *out = new (std::nothrow) fs_graph();
  if (!*out) return fail(FS_ERR_INVALID_ARG, "fs_graph_create: out of host memory");
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_graph_create");
}

void fs_graph_destroy(fs_graph* g) { delete g; }

fs_tensor fs_graph_input(fs_graph* g, int32_t dtype, int32_t rank, const int64_t* dims) try {
  clear_error();
  if (!g || !dims) return fail(FS_ERR_INVALID_ARG, "fs_graph_input: null argument");
  if (g->finalized) return fail(FS_ERR_INVALID_ARG, "fs_graph_input: graph is finalized");
  if (!valid_dtype(dtype)) return fail(FS_ERR_INVALID_ARG, "fs_graph_input: bad dtype %d", dtype);
  if (rank < 1 || rank > FS_MAX_RANK) return fail(FS_ERR_SHAPE, "fs_graph_input: rank %d outside 1..%d", rank, FS_MAX_RANK);
  Tensor t;
  t.dtype = dtype;
  t.rank = rank;
  int64_t n = 1;
  for (int i = 0; i < rank; ++i) {
    if (dims[i] < 1) return fail(FS_ERR_SHAPE, "fs_graph_input: extent %lld of axis %d (empty tensors are rejected)", (long long)dims[i], i);
    t.dims[i] = dims[i];
    n *= dims[i];
    if (n >= (int64_t(1) << 31)) return fail(FS_ERR_SHAPE, "fs_graph_input: 2^31 or more elements");
  }
  t.input_slot = (int32_t)g->inputs.size();
  g->tensors.push_back(t);
  g->inputs.push_back((int32_t)g->tensors.size() - 1);
  return (fs_tensor)g->tensors.size() - 1;
} catch (...) {
  return fs::fail_caught("fs_graph_input");
}

fs_tensor fs_graph_op(fs_graph* g, int32_t opcode, int32_t n_in, const fs_tensor* in, const void* attr, size_t attr_bytes) try {
  clear_error();
  if (!g || !in) return fail(FS_ERR_INVALID_ARG, "fs_graph_op: null argument");
  if (g->finalized) return fail(FS_ERR_INVALID_ARG, "fs_graph_op: graph is finalized");
  if (opcode < 0 || opcode >= FS_OPCODE_COUNT) return fail(FS_ERR_INVALID_ARG, "fs_graph_op: bad opcode %d", opcode);
  if (n_in != operand_count(opcode))
    return fail(FS_ERR_INVALID_ARG, "fs_graph_op(%s): %d operands given, %d needed", opcode_name(opcode), n_in, operand_count(opcode));
  const int32_t next_id = (int32_t)g->tensors.size();
  for (int i = 0; i < n_in; ++i) {
    if (in[i] < 0) return fail(FS_ERR_INVALID_ARG, "fs_graph_op(%s): operand %d is an error code (%d)", opcode_name(opcode), i, in[i]);
    if (in[i] >= next_id)
      return fail(FS_ERR_CYCLE, "fs_graph_op(%s): operand %d (id %d) does not precede the op: cyclic or unknown", opcode_name(opcode), i, in[i]);
  }
  Op op;
  op.opcode = opcode;
  op.n_in = n_in;
  for (int i = 0; i < n_in; ++i) op.in[i] = in[i];
  const Tensor& a = g->tensors[in[0]];
  Tensor r;
  r.dtype = FS_F32;

  auto need_attr = [&](size_t bytes) -> bool { return attr != nullptr && attr_bytes >= bytes; };
  const bool is_transpose = opcode == FS_TRANSPOSE;
  for (int i = 0; i < n_in; ++i) {
    const int32_t dt = g->tensors[in[i]].dtype;
    if (!float_dtype(dt) && !is_transpose)
      return fail(FS_ERR_DTYPE, "fs_graph_op(%s): operand %d has dtype %s; only transpose moves integer tensors", opcode_name(opcode), i, dtype_name(dt));
  }

  if (opcode <= FS_MAX) {
    const Tensor& b = g->tensors[in[1]];
    r.rank = a.rank > b.rank ? a.rank : b.rank;
    for (int k = 0; k < r.rank; ++k) {
      const int ka = k - (r.rank - a.rank), kb = k - (r.rank - b.rank);
      const int64_t da = ka >= 0 ? a.dims[ka] : 1, db = kb >= 0 ? b.dims[kb] : 1;
      if (da != db && da != 1 && db != 1)
        return fail(FS_ERR_SHAPE, "fs_graph_op(%s): extents %lld and %lld do not broadcast (result axis %d)", opcode_name(opcode), (long long)da, (long long)db, k);
      r.dims[k] = da > db ? da : db;
    }
  } else if (opcode == FS_SCALE || opcode == FS_ADD_SCALAR) {
    if (!need_attr(sizeof(fs_attr_scalar))) return fail(FS_ERR_INVALID_ARG, "fs_graph_op(%s): needs fs_attr_scalar", opcode_name(opcode));
    op.scalar = static_cast<const fs_attr_scalar*>(attr)->value;
    r.rank = a.rank;
    memcpy(r.dims, a.dims, sizeof r.dims);
  } else if (opcode == FS_BROADCAST) {
    if (!need_attr(sizeof(fs_attr_dims))) return fail(FS_ERR_INVALID_ARG, "fs_graph_op(broadcast): needs fs_attr_dims");
    const fs_attr_dims* d = static_cast<const fs_attr_dims*>(attr);
    if (d->rank < a.rank || d->rank > FS_MAX_RANK) return fail(FS_ERR_SHAPE, "fs_graph_op(broadcast): target rank %d", d->rank);
    r.rank = d->rank;
    for (int k = 0; k < r.rank; ++k) {
      const int ka = k - (r.rank - a.rank);
      const int64_t da = ka >= 0 ? a.dims[ka] : 1;
      if (d->dims[k] < 1 || (da != 1 && da != d->dims[k]))
        return fail(FS_ERR_SHAPE, "fs_graph_op(broadcast): extent %lld cannot stretch to %lld (axis %d)", (long long)da, (long long)d->dims[k], k);
      r.dims[k] = d->dims[k];
    }
  } else if (opcode == FS_REDUCE_SUM || opcode == FS_REDUCE_MAX || opcode == FS_REDUCE_MEAN) {
    if (!need_attr(sizeof(fs_attr_axis))) return fail(FS_ERR_INVALID_ARG, "fs_graph_op(%s): needs fs_attr_axis", opcode_name(opcode));
    op.axis = static_cast<const fs_attr_axis*>(attr)->axis;
    if (op.axis < 0 || op.axis >= a.rank) return fail(FS_ERR_SHAPE, "fs_graph_op(%s): axis %d outside rank %d", opcode_name(opcode), op.axis, a.rank);
    r.rank = a.rank;
    memcpy(r.dims, a.dims, sizeof r.dims);
    r.dims[op.axis] = 1;
  } else if (opcode == FS_TRANSPOSE) {
    if (!need_attr(sizeof(int32_t) * (size_t)a.rank)) return fail(FS_ERR_INVALID_ARG, "fs_graph_op(transpose): needs fs_attr_perm");
    const int32_t* perm = static_cast<const fs_attr_perm*>(attr)->perm;
    bool seen[FS_MAX_RANK] = {false, false, false, false};
    r.rank = a.rank;
    r.dtype = a.dtype;
    for (int k = 0; k < a.rank; ++k) {
      if (perm[k] < 0 || perm[k] >= a.rank || seen[perm[k]]) return fail(FS_ERR_SHAPE, "fs_graph_op(transpose): perm is not a permutation");
      seen[perm[k]] = true;
      op.perm[k] = perm[k];
      r.dims[k] = a.dims[perm[k]];
    }
  } else if (opcode == FS_CONVERT) {
    if (!need_attr(sizeof(fs_attr_dtype))) return fail(FS_ERR_INVALID_ARG, "fs_graph_op(convert): needs fs_attr_dtype");
    op.to_dtype = static_cast<const fs_attr_dtype*>(attr)->dtype;
    if (!float_dtype(op.to_dtype)) return fail(FS_ERR_DTYPE, "fs_graph_op(convert): target dtype %d is not a float type", op.to_dtype);
    r.rank = a.rank;
    r.dtype = op.to_dtype;
    memcpy(r.dims, a.dims, sizeof r.dims);
  } else {  // plain unary
    r.rank = a.rank;
    memcpy(r.dims, a.dims, sizeof r.dims);
  }
  if (r.numel() >= (int64_t(1) << 31)) return fail(FS_ERR_SHAPE, "fs_graph_op(%s): result has 2^31 or more elements", opcode_name(opcode));

  r.producer = (int32_t)g->ops.size();
  op.out = next_id;
  for (int i = 0; i < n_in; ++i) g->tensors[in[i]].consumers.push_back(r.producer);
  g->tensors.push_back(r);
  g->ops.push_back(op);
  return next_id;
} catch (...) {
  return fs::fail_caught("fs_graph_op");
}

fs_status fs_graph_output(fs_graph* g, fs_tensor t, int32_t store_as) try {
  clear_error();
  if (!g) return fail(FS_ERR_INVALID_ARG, "fs_graph_output: graph is null");
  if (g->finalized) return fail(FS_ERR_INVALID_ARG, "fs_graph_output: graph is finalized");
  if (t < 0 || t >= (int32_t)g->tensors.size()) return fail(FS_ERR_INVALID_ARG, "fs_graph_output: bad tensor id %d", t);
  if (!valid_dtype(store_as)) return fail(FS_ERR_INVALID_ARG, "fs_graph_output: bad dtype %d", store_as);
  Tensor& x = g->tensors[t];
  if (x.output_slot >= 0) return fail(FS_ERR_INVALID_ARG, "fs_graph_output: tensor %d is already an output", t);
  if (x.producer < 0) return fail(FS_ERR_INVALID_ARG, "fs_graph_output: tensor %d is a graph input", t);
  if ((x.dtype == FS_I32) != (store_as == FS_I32))
    return fail(FS_ERR_DTYPE, "fs_graph_output: %s tensor cannot be stored as %s", dtype_name(x.dtype), dtype_name(store_as));
  if (g->ops[x.producer].opcode == FS_TRANSPOSE && store_as != x.dtype)
    return fail(FS_ERR_DTYPE, "fs_graph_output: a transpose result keeps its dtype (%s)", dtype_name(x.dtype));
  x.output_slot = (int32_t)g->outputs.size();
  x.store_as = store_as;
  g->outputs.push_back(t);
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_graph_output");
}

fs_status fs_graph_external(fs_graph* g, fs_tensor from, fs_tensor input) try {
  clear_error();
  if (!g) return fail(FS_ERR_INVALID_ARG, "fs_graph_external: graph is null");
  if (g->finalized) return fail(FS_ERR_INVALID_ARG, "fs_graph_external: graph is finalized");
  const int32_t n = (int32_t)g->tensors.size();
  if (from < 0 || from >= n || input < 0 || input >= n) return fail(FS_ERR_INVALID_ARG, "fs_graph_external: bad tensor id");
  if (g->tensors[from].producer < 0) return fail(FS_ERR_INVALID_ARG, "fs_graph_external: tensor %d is not the result of an op", from);
  if (g->tensors[input].producer >= 0) return fail(FS_ERR_INVALID_ARG, "fs_graph_external: tensor %d is not a graph input", input);
  // declared before anything reads the input: the order in which ops were added stays an order of execution
  if (!g->tensors[input].consumers.empty())
    return fail(FS_ERR_INVALID_ARG, "fs_graph_external: input %d is already read by an op; declare the dependence first", input);
  g->external.emplace_back(from, input);
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_graph_external");
}

fs_status fs_graph_finalize(fs_graph* g) try {
  clear_error();
  if (!g) return fail(FS_ERR_INVALID_ARG, "fs_graph_finalize: graph is null");
  if (g->finalized) return FS_OK;
  if (g->outputs.empty()) return fail(FS_ERR_INVALID_ARG, "fs_graph_finalize: no output declared");
  for (const std::pair<int32_t, int32_t>& e : g->external)
    if (g->tensors[e.first].output_slot < 0)
      return fail(FS_ERR_INVALID_ARG, "fs_graph_finalize: tensor %d feeds an external computation and must be a graph output", e.first);
  // every op must reach an output (no dead code inside a fusion pattern)
  for (const Op& op : g->ops) {
    const Tensor& t = g->tensors[op.out];
    if (t.output_slot < 0 && t.consumers.empty())
      return fail(FS_ERR_INVALID_ARG, "fs_graph_finalize: result of op %s (tensor %d) is neither consumed nor an output", opcode_name(op.opcode), op.out);
  }
  g->finalized = true;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_graph_finalize");
}

}  // extern "C"

std::vector<std::vector<int>> fs_graph::external_producers() const {
  std::vector<std::vector<int>> waits(ops.size());
  for (const std::pair<int32_t, int32_t>& e : external)
    for (int32_t reader : tensors[e.second].consumers) waits[reader].push_back(tensors[e.first].producer);
  for (std::vector<int>& w : waits) {
    std::sort(w.begin(), w.end());
    w.erase(std::unique(w.begin(), w.end()), w.end());
  }
  return waits;
}
