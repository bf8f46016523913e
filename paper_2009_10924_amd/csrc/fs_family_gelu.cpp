// Pattern family: bias + GELU, alone or with the bias gradient (column reduction, global hand-off), and the fold launch.
#include "fs_stitch_util.hpp"

namespace fs {

void make_fold_launch(Launch* f, uint32_t n_rows, uint32_t width, uint32_t split, uint32_t stride, int32_t out_dt) {
  f->kernel = K_COLFOLD;
  GeluP fp{};
  fp.dt = out_dt;
  fp.n_row_tiles = n_rows;
  fp.cols = stride ? stride : width;   // distance between partial rows (a fold may take a slice of wider rows)
  fp.fold_cols = width;
  fp.fold_split = split;
  fp.fold_quads = n_rows > 128 ? 4 : 16;
  f->args.u.gelu = fp;
  f->shape.block[0] = 256;
  f->shape.grid[0] = (width / 4 + fp.fold_quads - 1) / fp.fold_quads;
}

// ------------------------------------------------------------------ bias-GELU family
bool build_gelu(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  MatchState st;
  bool with_dbias = false;
  if (g.outputs.size() == 2) {
    Pattern py("gelu(add($X,$B))"), pd("rsum[-2](mul($G,gelugrad(add($X,$B))))");
    int32_t ty = g.outputs[0], td = g.outputs[1];
    MatchState trial;
    if (!(py.match(g, ty, &trial) && pd.match(g, td, &trial))) {
      trial = MatchState();
      std::swap(ty, td);
      if (!(py.match(g, ty, &trial) && pd.match(g, td, &trial))) return false;
    }
    if (!covers_all(g, trial)) return false;
    st = trial;
    st.tensors["__y"] = ty;
    st.tensors["__d"] = td;
    with_dbias = true;
  } else if (g.outputs.size() == 1) {
    Pattern py("gelu(add($X,$B))");
    if (!py.match(g, g.outputs[0], &st) || !covers_all(g, st)) return false;
    st.tensors["__y"] = g.outputs[0];
  } else {
    return false;
  }
  int32_t tx = st.tensors["X"], tb = st.tensors["B"];
  if (!is_input(g, tx) || !is_input(g, tb)) return false;
  if (g.tensors[tx].numel() < g.tensors[tb].numel()) std::swap(tx, tb);
  const Tensor& x = g.tensors[tx];
  if (x.rank != 2 && with_dbias) return true;
  GeluP p{};
  p.cols = (uint32_t)x.dims[x.rank - 1];
  p.rows = (uint32_t)(x.numel() / p.cols);
  p.dt = x.dtype;
  p.bias_dt = g.tensors[tb].dtype;
  const Tensor& y = g.tensors[st.tensors["__y"]];
  if (!is_row_vector(g.tensors[tb], p.cols) || p.bias_dt != p.dt || y.store_as != p.dt) return true;
  const int VEC = vec_of(p.dt);
  if (p.cols % VEC != 0) return true;
  const int esz = dtype_bytes(p.dt);
  const double n = (double)p.rows * p.cols;

  if (!with_dbias) {
    pack->spec = PACK_BIAS_GELU;
    pack->in_dt = pack->out_dt = p.dt;
    pack->rows = p.rows;
    pack->cols = p.cols;
    pack->in_slot[0] = slot_of(g, tx);
    pack->vec_slot[0] = slot_of(g, tb);
    Candidate c = make_candidate(g, "bias_gelu", FS_SCHEME_LOCAL, K_BIAS_GELU);
    Launch& l = c.launches.front();
    l.args.u.gelu = p;
    l.ptr[0] = in_ref(g, tx);
    l.ptr[1] = in_ref(g, tb);
    l.ptr[2] = out_ref(0);
    l.shape.block[0] = 256;
    l.shape.grid[0] = (uint32_t)((n / VEC + 255) / 256);
    c.info.vecs_per_lane = 1;
    KernelCost kc;
    kc.hbm_bytes = 2 * n * esz + p.cols * esz;
    kc.elems = n;
    kc.valu_per_elem = 10 + (esz == 2 ? 2 : 0);
    kc.trans_per_elem = 2;
    kc.waves = (double)l.shape.grid[0] * 4;
    kc.waves_per_block = 4;
    kc.bytes_in_flight_per_lane = 16;
    kc.vgpr_estimate = 24;
    char var[24];
    snprintf(var, sizeof var, "<%s>", dtype_name(p.dt));
    finish_candidate(&c, var, kc);
    out->push_back(c);
    return true;
  }

  const int32_t tg = st.tensors["G"];
  const Tensor& d = g.tensors[st.tensors["__d"]];
  if (!is_input(g, tg) || !same_dims(g.tensors[tg], x) || g.tensors[tg].dtype != p.dt || d.store_as != FS_F32) return true;
  const uint32_t tile_cols = 64 * VEC;
  const uint32_t n_col_tiles = (p.cols + tile_cols - 1) / tile_cols;
  struct Shape { int waves, unroll; };
  {
    for (Shape sh : {Shape{4, 2}, Shape{4, 4}, Shape{8, 2}, Shape{8, 4}}) {
      const uint32_t tile_rows = sh.waves * sh.unroll;
      const uint32_t max_rb = (p.rows + tile_rows - 1) / tile_rows;
      uint32_t last_rb = 0;
      for (uint32_t want : {128u, 256u}) {
        // enough workgroups to fill the chip, few enough that the partials stay small
        const uint32_t n_rb = std::min(max_rb, std::max<uint32_t>(1, want * 6 / n_col_tiles));
        if (n_rb == last_rb) continue;
        last_rb = n_rb;
        Candidate c = make_candidate(g, "bias_gelu_dbias", FS_SCHEME_GLOBAL, K_BIAS_GELU_DBIAS);
        GeluP q = p;
        q.n_row_tiles = n_rb;
        q.waves = sh.waves;
        q.unroll = sh.unroll;
        q.fast = (p.rows % (n_rb * tile_rows) == 0 && p.cols % tile_cols == 0) ? 1 : 0;
        {
          Launch& l = c.launches.front();
          l.args.u.gelu = q;
          l.ptr[0] = in_ref(g, tx);
          l.ptr[1] = in_ref(g, tb);
          l.ptr[2] = in_ref(g, tg);
          l.ptr[3] = out_ref(y.output_slot);
          l.ptr[4] = ws_ref(0);
          l.shape.block[0] = sh.waves * 64;
          l.shape.grid[0] = n_rb * n_col_tiles;
        }
        {
          // the global hand-off: a second launch folds the row blocks' partial sums
          c.launches.emplace_back();
          Launch& f = c.launches.back();
          make_fold_launch(&f, n_rb, p.cols, p.cols);
          f.ptr[0] = ws_ref(0);
          f.ptr[1] = out_ref(d.output_slot);
          c.info.n_kernels = 2;
        }
        c.info.workspace_bytes = (int64_t)n_rb * p.cols * 4;
        c.info.rows_per_block = (int32_t)tile_rows;
        c.info.vecs_per_lane = sh.unroll;
        c.info.lanes_per_row = 64;
        c.info.lds_bytes = sh.waves * (int32_t)tile_cols * 4 + 4;
        c.info.bytes_moved_model = c.info.bytes_min + 2ll * n_rb * p.cols * 4;
        KernelCost kc;
        kc.hbm_bytes = 3 * n * esz + 2.0 * n_rb * p.cols * 4;
        kc.elems = n;
        kc.valu_per_elem = 13 + (esz == 2 ? 1 : 0);
        kc.trans_per_elem = 2;
        kc.waves_per_block = sh.waves;
        kc.waves = (double)n_rb * n_col_tiles * sh.waves;
        kc.bytes_in_flight_per_lane = 32.0 * sh.unroll;
        kc.vgpr_estimate = 40 + 16 * sh.unroll;
        kc.barriers = 1;
        kc.lds_bytes_per_block = c.info.lds_bytes;
        kc.rows_per_wave_loop = std::max(1.0, (double)p.rows / ((double)n_rb * tile_rows));
        kc.dep_phases = 0;   // software pipelined: only the first tile's load latency is exposed (added below)
        // the fold: a second launch spread over the chip
        kc.serial_tail_s = device().mem_latency_s + 0.5 * device().launch_s + device().mem_latency_s * std::ceil(n_rb / 16.0 / 8.0) * 0.5;
        char var[48];
        snprintf(var, sizeof var, "<%s,W%d,U%d,RB%u,fold>", dtype_name(p.dt), sh.waves, sh.unroll, n_rb);
        finish_candidate(&c, var, kc);
        out->push_back(c);
      }
    }
  }
  return true;
}

}  // namespace fs
