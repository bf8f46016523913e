// Per-op baseline plan: one launch per op in graph order (two for a reduction over
// a non-innermost axis), float32 intermediates in the caller's workspace.
#include <algorithm>
#include <cstring>

#include "fs_internal.hpp"

namespace fs {

namespace {

constexpr int64_t kAlign = 256;
int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// First-fit reuse of workspace blocks whose tenant is dead (lifetime = producer op
// to last consumer op).  A block is never handed to the op that still reads it.
struct Arena {
  struct Block { int64_t off, size; bool free; };
  std::vector<Block> blocks;
  int64_t top = 0;
  int64_t alloc(int64_t bytes) {
    bytes = round_up(bytes, kAlign);
    for (Block& b : blocks)
      if (b.free && b.size >= bytes) { b.free = false; return b.off; }
    blocks.push_back({top, bytes, false});
    top += bytes;
    return top - bytes;
  }
  void release(int64_t off) {
    for (Block& b : blocks)
      if (b.off == off) b.free = true;
  }
};

int pick_vec(int64_t inner) { return inner % 8 == 0 ? 8 : inner % 4 == 0 ? 4 : 1; }

uint32_t pow2_at_least(uint32_t v) {
  uint32_t p = 1;
  while (p < v) p <<= 1;
  return p;
}

}  // namespace

fs_status build_unfused(const fs_graph& g, Candidate* out) {
  const int n_t = (int)g.tensors.size();
  std::vector<BufRef> where(n_t);
  std::vector<int32_t> dt(n_t);          // dtype of the buffer that holds the tensor
  std::vector<int> last_use(n_t, -1);
  for (int t = 0; t < n_t; ++t)
    for (int c : g.tensors[t].consumers) last_use[t] = std::max(last_use[t], c);

  for (int t : g.inputs) {
    where[t].kind = BUF_INPUT;
    where[t].slot = g.tensors[t].input_slot;
    dt[t] = g.tensors[t].dtype;
  }

  Arena arena;
  int64_t moved = 0;
  std::vector<Launch>& L = out->launches;
  L.clear();

  auto add_launch = [&](int32_t kernel) -> Launch& {
    L.emplace_back();
    L.back().kernel = kernel;
    L.back().shape.block[0] = 256;
    return L.back();
  };
  auto grid1d = [](Launch& l, int64_t threads) { l.shape.grid[0] = (uint32_t)std::max<int64_t>(1, (threads + 255) / 256); };

  for (int oi = 0; oi < (int)g.ops.size(); ++oi) {
    const Op& op = g.ops[oi];
    const Tensor& r = g.tensors[op.out];
    const Tensor& a = g.tensors[op.in[0]];
    const int64_t n_out = r.numel();

    // where the result lives
    BufRef dst;
    int32_t dst_dt = r.dtype;
    bool extra_store = false;   // output with consumers and a narrower storage dtype
    if (r.output_slot >= 0 && (r.consumers.empty() || r.store_as == r.dtype)) {
      dst.kind = BUF_OUTPUT;
      dst.slot = r.output_slot;
      dst_dt = r.store_as;
    } else {
      dst.kind = BUF_WORKSPACE;
      dst.offset = arena.alloc(n_out * dtype_bytes(r.dtype));
      extra_store = r.output_slot >= 0;
    }
    where[op.out] = dst;
    dt[op.out] = dst_dt;

    const int32_t opc = op.opcode;
    if (opc <= FS_MAX || opc == FS_BROADCAST) {
      const int ib = opc == FS_BROADCAST ? op.in[0] : op.in[1];
      const Tensor& b = g.tensors[ib];
      // per-axis strides of both operands over the result, then collapse
      int64_t dims[FS_MAX_RANK], sa[FS_MAX_RANK], sb[FS_MAX_RANK];
      auto strides = [&](const Tensor& t, int64_t* s) {
        int64_t acc = 1;
        for (int k = r.rank - 1; k >= 0; --k) {
          const int kt = k - (r.rank - t.rank);
          const int64_t d = kt >= 0 ? t.dims[kt] : 1;
          s[k] = (d == 1) ? 0 : acc;
          acc *= d;
        }
      };
      strides(a, sa);
      strides(b, sb);
      for (int k = 0; k < r.rank; ++k) dims[k] = r.dims[k];
      int64_t cd[FS_MAX_RANK], ca[FS_MAX_RANK], cb[FS_MAX_RANK];
      int cr = 0;
      for (int k = 0; k < r.rank; ++k) {
        if (dims[k] == 1) continue;
        if (cr > 0 && ca[cr - 1] == sa[k] * dims[k] && cb[cr - 1] == sb[k] * dims[k]) {
          cd[cr - 1] *= dims[k];
          ca[cr - 1] = sa[k];
          cb[cr - 1] = sb[k];
        } else {
          cd[cr] = dims[k]; ca[cr] = sa[k]; cb[cr] = sb[k];
          ++cr;
        }
      }
      if (cr == 0) { cd[0] = 1; ca[0] = 0; cb[0] = 0; cr = 1; }
      Launch& l = add_launch(K_BINARY);
      BinaryP& p = l.args.u.binary;
      p = BinaryP{};
      p.op = opc == FS_BROADCAST ? B_FIRST : opc;   // B_ADD..B_MAX share the opcode numbering
      p.a_dt = dt[op.in[0]]; p.b_dt = dt[ib]; p.out_dt = dst_dt;
      p.rank = cr;
      p.n = (uint32_t)n_out;
      for (int k = 0; k < cr; ++k) { p.dims[k] = (uint32_t)cd[k]; p.sa[k] = (uint32_t)ca[k]; p.sb[k] = (uint32_t)cb[k]; }
      p.vec = pick_vec(cd[cr - 1]);
      l.ptr[0] = where[op.in[0]]; l.ptr[1] = where[ib]; l.ptr[2] = dst;
      grid1d(l, n_out / p.vec);
      moved += a.numel() * dtype_bytes(p.a_dt) + (opc == FS_BROADCAST ? 0 : b.numel() * dtype_bytes(p.b_dt)) + n_out * dtype_bytes(dst_dt);
    } else if (opc == FS_REDUCE_SUM || opc == FS_REDUCE_MAX || opc == FS_REDUCE_MEAN) {
      int64_t outer = 1, inner = 1;
      for (int k = 0; k < op.axis; ++k) outer *= a.dims[k];
      for (int k = op.axis + 1; k < a.rank; ++k) inner *= a.dims[k];
      const int64_t red = a.dims[op.axis];
      const int32_t rop = opc == FS_REDUCE_SUM ? R_SUM : opc == FS_REDUCE_MAX ? R_MAX : R_MEAN;
      const float mean_scale = rop == R_MEAN ? (float)(1.0 / (double)red) : 1.0f;
      if (inner == 1) {
        Launch& l = add_launch(K_REDUCE_ROW);
        ReduceP& p = l.args.u.reduce;
        p = ReduceP{};
        p.op = rop; p.in_dt = dt[op.in[0]]; p.out_dt = dst_dt;
        p.outer = (uint32_t)outer; p.red = (uint32_t)red; p.inner = 1;
        p.vec = pick_vec(red);
        p.lanes_per_row = std::min<uint32_t>(64, pow2_at_least((uint32_t)((red + p.vec - 1) / p.vec)));
        p.post_scale = mean_scale;
        l.ptr[0] = where[op.in[0]]; l.ptr[1] = dst;
        l.shape.grid[0] = (uint32_t)((outer + 256 / p.lanes_per_row - 1) / (256 / p.lanes_per_row));
      } else {
        const int vec = pick_vec(inner);
        const int64_t inner_blocks = (inner / vec + 255) / 256;
        int64_t nchunk = std::max<int64_t>(1, 2048 / std::max<int64_t>(1, outer * inner_blocks));
        nchunk = std::min<int64_t>(nchunk, std::max<int64_t>(1, red / 32));
        const int64_t chunk = (red + nchunk - 1) / nchunk;
        nchunk = (red + chunk - 1) / chunk;
        BufRef partial = dst;
        int32_t partial_dt = dst_dt;
        if (nchunk > 1) {
          partial.kind = BUF_WORKSPACE;
          partial.offset = arena.alloc(outer * nchunk * inner * 4);
          partial_dt = FS_F32;
        }
        {
          Launch& l = add_launch(K_REDUCE_MID);
          ReduceP& p = l.args.u.reduce;
          p = ReduceP{};
          p.op = rop; p.in_dt = dt[op.in[0]]; p.out_dt = partial_dt; p.vec = vec;
          p.outer = (uint32_t)outer; p.red = (uint32_t)red; p.inner = (uint32_t)inner;
          p.chunk = (uint32_t)chunk; p.nchunk = (uint32_t)nchunk;
          p.post_scale = nchunk > 1 ? 1.0f : mean_scale;
          l.ptr[0] = where[op.in[0]]; l.ptr[1] = partial;
          l.shape.grid[0] = (uint32_t)(inner_blocks * nchunk * outer);
        }
        if (nchunk > 1) {
          Launch& l = add_launch(K_REDUCE_MID);
          ReduceP& p = l.args.u.reduce;
          p = ReduceP{};
          p.op = rop == R_MEAN ? R_SUM : rop; p.in_dt = FS_F32; p.out_dt = dst_dt; p.vec = vec;
          p.outer = (uint32_t)outer; p.red = (uint32_t)nchunk; p.inner = (uint32_t)inner;
          p.chunk = (uint32_t)nchunk; p.nchunk = 1;
          p.post_scale = mean_scale;
          l.ptr[0] = partial; l.ptr[1] = dst;
          l.shape.grid[0] = (uint32_t)(inner_blocks * outer);
          arena.release(partial.offset);
          moved += 2 * outer * nchunk * inner * 4;
        }
      }
      moved += a.numel() * dtype_bytes(dt[op.in[0]]) + n_out * dtype_bytes(dst_dt);
    } else if (opc == FS_TRANSPOSE) {
      const int pad = FS_MAX_RANK - a.rank;
      int64_t in_stride_axis[FS_MAX_RANK];   // contiguous strides of the input, by input axis
      {
        int64_t acc = 1;
        for (int k = a.rank - 1; k >= 0; --k) { in_stride_axis[k] = acc; acc *= a.dims[k]; }
      }
      const bool keeps_inner = op.perm[a.rank - 1] == a.rank - 1;
      Launch& l = add_launch(keeps_inner ? K_TRANSPOSE_ROWS : K_TRANSPOSE_TILE);
      TransposeP& p = l.args.u.transpose;
      p = TransposeP{};
      p.elem_bytes = dtype_bytes(a.dtype);
      p.n = (uint32_t)n_out;
      for (int k = 0; k < FS_MAX_RANK; ++k) { p.out_dims[k] = 1; p.in_stride[k] = 0; p.out_stride[k] = 0; }
      {
        int64_t acc = 1;
        for (int k = r.rank - 1; k >= 0; --k) {
          p.out_dims[pad + k] = (uint32_t)r.dims[k];
          p.in_stride[pad + k] = (uint32_t)in_stride_axis[op.perm[k]];
          p.out_stride[pad + k] = (uint32_t)acc;
          acc *= r.dims[k];
        }
      }
      l.ptr[0] = where[op.in[0]]; l.ptr[1] = dst;
      if (keeps_inner) {
        const int64_t inner = r.dims[r.rank - 1];
        const int max_vec = 16 / p.elem_bytes;
        int vec = max_vec;
        while (vec > 1 && inner % vec != 0) vec >>= 1;
        p.vec = vec;
        grid1d(l, n_out / vec);
      } else {
        uint32_t q = 0;
        for (int k = 0; k < r.rank; ++k) if (op.perm[k] == a.rank - 1) q = (uint32_t)(pad + k);
        p.tile_in_axis_out_pos = q;
        // both tile axes multiples of a 128-bit vector: 64x64 tile with vector accesses, else 32x32 scalar
        const uint32_t v128 = 16 / p.elem_bytes;
        p.vec = (p.out_dims[q] % v128 == 0 && p.out_dims[3] % v128 == 0) ? (int32_t)v128 : 1;
        // vectorised tile: 16 x 16 units of vec x vec elements, or 8 x 32 when the moving axis is short
        // neighbouring workgroups: when the inner axis outside the tile follows the tile's rows directly in the input
        // ([B,S,H,D] -> [B,H,D,S]: a head's 64 x D tile is followed by the next head's), walking that axis first makes
        // neighbours read one contiguous span (measured: 3 % on float32, nothing on 16-bit elements)
        {
          uint32_t ax1 = 0;
          for (uint32_t k = 0; k < 3; ++k) if (k != q) ax1 = k;
          p.order = (p.out_dims[ax1] > 1 && p.in_stride[ax1] == p.out_dims[q]) ? 1u : 0u;
        }
        p.tile_uq = p.vec > 1 ? (p.out_dims[q] > 8u * (uint32_t)p.vec ? 16u : 8u) : 0u;
        const int64_t tile_q = p.vec > 1 ? (int64_t)p.tile_uq * p.vec : 32, tile_3 = p.vec > 1 ? (int64_t)(256 / p.tile_uq) * p.vec : 32;
        int64_t blocks = ((int64_t)p.out_dims[q] + tile_q - 1) / tile_q * (((int64_t)p.out_dims[3] + tile_3 - 1) / tile_3);
        for (uint32_t k = 0; k < 3; ++k) if (k != q) blocks *= p.out_dims[k];
        if (blocks >= (int64_t(1) << 31)) return fail(FS_ERR_SHAPE, "transpose: too many tiles");
        l.shape.grid[0] = (uint32_t)blocks;
      }
      moved += 2 * n_out * p.elem_bytes;
    } else {
      // unary family, convert included
      Launch& l = add_launch(K_UNARY);
      UnaryP& p = l.args.u.unary;
      p = UnaryP{};
      switch (opc) {
        case FS_SCALE: p.op = U_SCALE; break;
        case FS_ADD_SCALAR: p.op = U_ADD_SCALAR; break;
        case FS_SQUARE: p.op = U_SQUARE; break;
        case FS_EXP: p.op = U_EXP; break;
        case FS_RSQRT: p.op = U_RSQRT; break;
        case FS_TANH: p.op = U_TANH; break;
        case FS_GELU_TANH: p.op = U_GELU; break;
        case FS_GELU_TANH_GRAD: p.op = U_GELU_GRAD; break;
        case FS_LOG: p.op = U_LOG; break;
        case FS_SIGMOID: p.op = U_SIGMOID; break;
        case FS_RELU: p.op = U_RELU; break;
        case FS_ABS: p.op = U_ABS; break;
        case FS_SQRT: p.op = U_SQRT; break;
        default: p.op = U_COPY; break;   // FS_CONVERT: the store does the rounding
      }
      p.in_dt = dt[op.in[0]]; p.out_dt = dst_dt;
      p.n = (uint32_t)n_out;
      p.vec = pick_vec(n_out);
      p.value = (float)op.scalar;
      l.ptr[0] = where[op.in[0]]; l.ptr[1] = dst;
      grid1d(l, n_out / p.vec);
      moved += n_out * (dtype_bytes(p.in_dt) + dtype_bytes(dst_dt));
    }

    if (extra_store) {
      Launch& l = add_launch(K_UNARY);
      UnaryP& p = l.args.u.unary;
      p = UnaryP{};
      p.op = U_COPY; p.in_dt = dst_dt; p.out_dt = r.store_as;
      p.n = (uint32_t)n_out; p.vec = pick_vec(n_out);
      l.ptr[0] = dst;
      l.ptr[1].kind = BUF_OUTPUT; l.ptr[1].slot = r.output_slot;
      grid1d(l, n_out / p.vec);
      moved += n_out * (dtype_bytes(dst_dt) + dtype_bytes(r.store_as));
    }

    // operands that die here give their workspace back
    for (int i = 0; i < op.n_in; ++i) {
      const int t = op.in[i];
      if (where[t].kind == BUF_WORKSPACE && last_use[t] == oi && !(i == 1 && op.in[0] == op.in[1])) arena.release(where[t].offset);
    }
  }

  fs_plan_info& info = out->info;
  memset(&info, 0, sizeof info);
  info.scheme = FS_SCHEME_UNFUSED;
  info.n_kernels = (int32_t)L.size();
  info.workspace_bytes = arena.top;
  info.bytes_min = graph_bytes_min(g);
  info.bytes_moved_model = moved;
  snprintf(info.pattern, sizeof info.pattern, "unfused");
  // dominant kernel = the launch with the most threads
  size_t dom = 0;
  for (size_t i = 1; i < L.size(); ++i)
    if ((uint64_t)L[i].shape.grid[0] > (uint64_t)L[dom].shape.grid[0]) dom = i;
  if (!L.empty()) {
    for (int k = 0; k < 3; ++k) { info.block[k] = (int32_t)L[dom].shape.block[k]; info.grid[k] = (int32_t)L[dom].shape.grid[k]; }
    snprintf(info.kernel, sizeof info.kernel, "%s", kernel_name(L[dom].kernel));
  }
  return FS_OK;
}

int64_t graph_bytes_min(const fs_graph& g) {
  int64_t b = 0;
  for (int t : g.inputs) b += g.tensors[t].numel() * dtype_bytes(g.tensors[t].dtype);
  for (int t : g.outputs) b += g.tensors[t].numel() * dtype_bytes(g.tensors[t].store_as);
  return b;
}

}  // namespace fs
