// Pattern families: residual add + bias + LayerNorm (forward, optionally with saved statistics) and LayerNorm backward.
#include "fs_stitch_util.hpp"

namespace fs {

// ------------------------------------------------------------------ layernorm family
bool build_layernorm(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  // one normalised output; a training forward pass may hand out the per-row mean and the reciprocal standard
  // deviation as well (two more outputs, float32 [rows, 1])
  if (g.outputs.empty() || g.outputs.size() > 3) return false;
  int32_t root = -1;
  for (int32_t t : g.outputs)
    if (root < 0 || g.tensors[t].numel() > g.tensors[root].numel()) root = t;
  static const char* hs[] = {"add(add($X,$R),$B)", "add($X,$R)", "$X"};
  const std::string c_txt = "sub(@,rmean[-1](@))";
  const std::string norm_txt = "mul(%,rsqrt(addc[#0](rmean[-1](square(%)))))";
  MatchState st;
  bool found = false, affine = false;
  for (const char* h : hs) {
    const std::string c = subst(c_txt, h);
    std::string norm;
    for (char ch : norm_txt) {
      if (ch == '%') norm += c;
      else norm += ch;
    }
    for (int variant = 0; variant < 4 && !found; ++variant) {
      std::string top = (variant & 1) ? norm : "add(mul(" + norm + ",$G),$Bt)";
      if (variant & 2) top = "cvt(" + top + ")";
      Pattern pat(top);
      MatchState trial;
      if (pat.match(g, root, &trial) && covers_all(g, trial)) {
        bool inputs_ok = true;
        for (auto& kv : trial.tensors) inputs_ok = inputs_ok && is_input(g, kv.second);
        if (inputs_ok) {
          st = trial;
          found = true;
          affine = !(variant & 1);
        }
      }
    }
    if (found) break;
  }
  if (!found) return false;

  int32_t tx = st.tensors["X"], tr = st.tensors.count("R") ? st.tensors["R"] : -1, tb = st.tensors.count("B") ? st.tensors["B"] : -1;
  // put the full-shaped tensor in X; a lone second operand is a residual or a bias by its shape
  auto full = [&](int32_t a, int32_t b) { return g.tensors[a].numel() >= g.tensors[b].numel(); };
  if (tr >= 0 && !full(tx, tr)) std::swap(tx, tr);
  const Tensor& x = g.tensors[tx];
  LayerNormP p{};
  p.cols = (uint32_t)x.dims[x.rank - 1];
  p.rows = (uint32_t)(x.numel() / p.cols);
  if (tr >= 0 && tb < 0 && !same_dims(g.tensors[tr], x)) { tb = tr; tr = -1; }
  if (tr >= 0 && !same_dims(g.tensors[tr], x)) return true;
  if (tb >= 0 && !is_row_vector(g.tensors[tb], p.cols)) return true;
  const int32_t tg = affine ? st.tensors["G"] : -1, tbt = affine ? st.tensors["Bt"] : -1;
  if (affine && (!is_row_vector(g.tensors[tg], p.cols) || !is_row_vector(g.tensors[tbt], p.cols))) return true;
  p.in_dt = x.dtype;
  p.par_dt = x.dtype;
  p.out_dt = g.tensors[root].store_as;
  // the other outputs: the row mean (the reduction whose result is subtracted) and the reciprocal standard
  // deviation (the rsqrt), stored as float32
  int32_t t_mean = -1, t_rstd = -1;
  for (int32_t t : g.outputs) {
    if (t == root) continue;
    const Tensor& T = g.tensors[t];
    if (T.store_as != FS_F32 || T.producer < 0 || T.numel() != (int64_t)p.rows) return true;
    const Op& maker = g.ops[T.producer];
    bool feeds_sub = false;
    for (int c : T.consumers) feeds_sub = feeds_sub || g.ops[c].opcode == FS_SUB;
    if (maker.opcode == FS_RSQRT && t_rstd < 0) t_rstd = t;
    else if (maker.opcode == FS_REDUCE_MEAN && feeds_sub && t_mean < 0) t_mean = t;
    else return true;
  }
  const bool with_stats = t_mean >= 0 || t_rstd >= 0;
  for (int32_t t : {tr, tb, tg, tbt})
    if (t >= 0 && g.tensors[t].dtype != x.dtype) return true;
  if (!(p.in_dt == FS_F32 || p.out_dt == p.in_dt)) return true;   // compiled dtype pairs
  p.has_res = tr >= 0;
  p.has_bias = tb >= 0;
  p.has_affine = affine;
  p.stats = with_stats ? 1 : 0;
  p.eps = (float)st.scalars[0];
  p.inv_cols = (float)(1.0 / (double)p.cols);

  const int VEC = vec_of(p.in_dt);
  if (p.cols % VEC != 0) return true;
  const uint32_t nvec = p.cols / VEC;
  const int in_b = dtype_bytes(p.in_dt), out_b = dtype_bytes(p.out_dt);
  const double n = (double)p.rows * p.cols;
  const int n_vec_inputs = (p.has_bias ? 1 : 0) + (affine ? 2 : 0);
  if (!with_stats && affine && p.has_res == p.has_bias && (p.out_dt == p.in_dt || p.out_dt == FS_BF16)) {
    pack->spec = p.has_res ? PACK_LN_FULL : PACK_LN_PLAIN;
    pack->in_dt = p.in_dt;
    pack->out_dt = p.out_dt;
    pack->rows = p.rows;
    pack->cols = p.cols;
    pack->f[0] = p.eps;
    pack->f[1] = p.inv_cols;
    pack->in_slot[0] = slot_of(g, tx);
    if (p.has_res) {
      pack->in_slot[1] = slot_of(g, tr);
      pack->vec_slot[0] = slot_of(g, tb);
      pack->vec_slot[1] = slot_of(g, tg);
      pack->vec_slot[2] = slot_of(g, tbt);
    } else {
      pack->vec_slot[0] = slot_of(g, tg);
      pack->vec_slot[1] = slot_of(g, tbt);
    }
  }
  auto base_cost = [&](KernelCost* kc) {
    kc->hbm_bytes = n * in_b * (1 + p.has_res) + n * out_b + (double)n_vec_inputs * p.cols * in_b +
                    4.0 * p.rows * ((t_mean >= 0) + (t_rstd >= 0));
    kc->elems = n;
    kc->valu_per_elem = 8.0 + (in_b == 2 ? 1.0 : 0.0) + (out_b == 2 ? 1.0 : 0.0);
    kc->trans_per_elem = 0.0;
    kc->dep_phases = 1;
  };
  auto fill_ptrs = [&](Launch& l) {
    l.ptr[0] = in_ref(g, tx);
    if (tr >= 0) l.ptr[1] = in_ref(g, tr);
    if (tb >= 0) l.ptr[2] = in_ref(g, tb);
    if (affine) { l.ptr[3] = in_ref(g, tg); l.ptr[4] = in_ref(g, tbt); }
    l.ptr[5] = out_ref(g.tensors[root].output_slot);
    if (t_mean >= 0) l.ptr[6] = out_ref(g.tensors[t_mean].output_slot);
    if (t_rstd >= 0) l.ptr[7] = out_ref(g.tensors[t_rstd].output_slot);
  };

  for (int K : {1, 2, 3, 4, 6, 8}) {
    const uint32_t L = pow2_at_least((nvec + K - 1) / K);
    if (L > 64) continue;
    if (K > 1 && (uint64_t)L * K >= 2ull * nvec) continue;
    Candidate c = make_candidate(g, "layernorm", L == 1 ? FS_SCHEME_LOCAL : FS_SCHEME_WAVE, K_LAYERNORM_WAVE);
    Launch& l = c.launches.front();
    LayerNormP q = p;
    q.lanes_per_row = (int32_t)L;
    q.lanes_log2 = log2_of(L);
    q.vecs_per_lane = K;
    q.rows_per_block = (int32_t)(256 / L);
    q.fast = p.has_res && p.has_bias && affine && (uint64_t)L * K == nvec && p.rows % (256 / L) == 0;
    l.args.u.layernorm = q;
    fill_ptrs(l);
    l.shape.block[0] = 256;
    l.shape.grid[0] = (p.rows + q.rows_per_block - 1) / q.rows_per_block;
    c.info.lanes_per_row = (int32_t)L;
    c.info.vecs_per_lane = K;
    c.info.rows_per_block = q.rows_per_block;
    KernelCost kc;
    base_cost(&kc);
    kc.waves = (double)l.shape.grid[0] * 4;
    kc.waves_per_block = 4;
    kc.bytes_in_flight_per_lane = 16.0 * K * (1 + p.has_res);
    kc.vgpr_estimate = 16 + K * (VEC + 8 + (affine ? 0 : 0)) + (K > 3 ? K * 4 : 0);
    int steps = 0;
    for (uint32_t s = 1; s < L; s <<= 1) ++steps;
    kc.xlane_steps = 2 * steps;
    kc.cache_bytes = n / p.cols * (double)n_vec_inputs * p.cols * in_b;   // bias/gamma/beta re-read per row from L1/L2
    kc.lane_utilisation = (double)nvec / ((double)L * K);
    kc.access_run_bytes = std::min<double>(L, nvec) * 16.0;
    char var[40];
    snprintf(var, sizeof var, "<%s,%s,K%d,L%u>", dtype_name(p.in_dt), dtype_name(p.out_dt), K, L);
    finish_candidate(&c, var, kc);
    out->push_back(c);
  }
  // block shapes: T threads (whole wavefronts) x K vectors per row.  Where some shape fills its lanes exactly, the
  // padded ones are not offered: their idle lanes still issue (clamped) loads and wait at the barriers (768 floats:
  // 192 threads x 1 vector measures 13.2 us, 128 threads x 2 vectors with a quarter of the lanes idle 14.9 us)
  auto block_threads = [&](int K) { return ((nvec + K - 1) / K + 63) / 64 * 64; };
  bool exact_fill_exists = false;
  for (int K : {1, 2, 3, 4, 6, 8}) {
    const uint32_t T = block_threads(K);
    exact_fill_exists = exact_fill_exists || (T >= 128 && T <= 256 && (uint64_t)T * K == nvec);
  }
  for (int K : {1, 2, 3, 4, 6, 8}) {
    const uint32_t T = block_threads(K);
    if (T > 256 || T < 128) continue;   // a single wave per row is the wave variant's job
    if ((uint64_t)T * K >= 2ull * nvec) continue;
    if (exact_fill_exists && (uint64_t)T * K != nvec) continue;
    Candidate c = make_candidate(g, "layernorm", FS_SCHEME_LDS, K_LAYERNORM_BLOCK);
    Launch& l = c.launches.front();
    LayerNormP q = p;
    q.lanes_per_row = (int32_t)T;
    q.vecs_per_lane = K;
    q.rows_per_block = 1;
    q.fast = !with_stats && p.has_res && p.has_bias && affine && (uint64_t)T * K == nvec;
    l.args.u.layernorm = q;
    fill_ptrs(l);
    l.shape.block[0] = T;
    // about 18 wavefronts per compute unit in one pass (measured on 8192 x 768 with 192 threads per row, workgroups
    // per CU -> us: 3 16.6, 4 14.6, 5 12.8, 6 11.9, 8 12.5, 10 13.0): fewer leave the memory pipeline idle between a
    // workgroup's rows, more only shorten each workgroup's walk
    const uint32_t blocks_per_cu = std::max<uint32_t>(1, (1152 + T / 2) / T);
    l.shape.grid[0] = std::min<uint32_t>(p.rows, device().n_cu * blocks_per_cu);
    c.info.lanes_per_row = (int32_t)T;
    c.info.vecs_per_lane = K;
    c.info.rows_per_block = 1;
    c.info.lds_bytes = 64;
    KernelCost kc;
    base_cost(&kc);
    kc.waves_per_block = T / 64;
    kc.waves = (double)l.shape.grid[0] * kc.waves_per_block;
    kc.rows_per_wave_loop = (double)p.rows / l.shape.grid[0];
    kc.bytes_in_flight_per_lane = 16.0 * K * (1 + p.has_res);
    kc.vgpr_estimate = 20 + K * VEC * 2;
    kc.xlane_steps = 12;
    kc.barriers = 2;
    kc.lds_bytes_per_block = 64;
    kc.cache_bytes = n / p.cols * (double)n_vec_inputs * p.cols * in_b;
    kc.lane_utilisation = (double)nvec / ((double)T * K);
    char var[40];
    snprintf(var, sizeof var, "<%s,%s,K%d,T%u>", dtype_name(p.in_dt), dtype_name(p.out_dt), K, T);
    finish_candidate(&c, var, kc);
    out->push_back(c);
  }
  return true;
}

// Fold launch of [n_rows, width] float32 column partials (see k_colfold).
// ------------------------------------------------------------------ layernorm backward
bool build_layernorm_backward(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  if (g.outputs.size() != 3) return false;
  const std::string xh = "mul(sub($H,$MU),$RS)", gg = "mul($DY,$G)";
  Pattern p_dx("mul(sub(sub(" + gg + ",rmean[-1](" + gg + ")),mul(" + xh + ",rmean[-1](mul(" + gg + "," + xh + ")))),$RS)");
  Pattern p_dg("rsum[-2](mul($DY," + xh + "))");
  Pattern p_db("rsum[-2]($DY)");
  MatchState st;
  int32_t t_dx = -1, t_dg = -1, t_db = -1;
  // dx binds every name; then the two column sums must agree with those bindings
  for (int32_t t : g.outputs)
    if (t_dx < 0 && p_dx.match(g, t, &st)) t_dx = t;
  if (t_dx < 0) return false;
  for (int32_t t : g.outputs) {
    if (t == t_dx) continue;
    if (t_dg < 0 && p_dg.match(g, t, &st)) { t_dg = t; continue; }
    if (t_db < 0 && p_db.match(g, t, &st)) { t_db = t; continue; }
  }
  if (t_dg < 0 || t_db < 0 || !covers_all(g, st)) return false;
  const int32_t th = st.tensors["H"], tdy = st.tensors["DY"], tg = st.tensors["G"], tmu = st.tensors["MU"], trs = st.tensors["RS"];
  for (int32_t t : {th, tdy, tg, tmu, trs})
    if (!is_input(g, t)) return false;
  const Tensor& h = g.tensors[th];
  if (h.rank != 2) return true;
  LnBwdP p{};
  p.rows = (uint32_t)h.dims[0];
  p.cols = (uint32_t)h.dims[1];
  p.dt = h.dtype;
  p.inv_cols = (float)(1.0 / (double)p.cols);
  const Tensor& mu = g.tensors[tmu];
  const Tensor& rs = g.tensors[trs];
  auto per_row = [&](const Tensor& t) { return t.rank == 2 && t.dims[0] == (int64_t)p.rows && t.dims[1] == 1 && t.dtype == FS_F32; };
  if (!same_dims(g.tensors[tdy], h) || g.tensors[tdy].dtype != p.dt || !is_row_vector(g.tensors[tg], p.cols) ||
      g.tensors[tg].dtype != p.dt || !per_row(mu) || !per_row(rs) || p.dt == FS_I32)
    return true;
  if (g.tensors[t_dx].store_as != p.dt || g.tensors[t_dg].store_as != FS_F32 || g.tensors[t_db].store_as != FS_F32) return true;
  const int VEC = vec_of(p.dt);
  if (p.cols % VEC != 0) return true;
  const uint32_t nvec = p.cols / VEC;
  const int esz = dtype_bytes(p.dt);
  const double n = (double)p.rows * p.cols;
  for (int K : {1, 2, 3, 4, 6}) {
    const uint32_t L = pow2_at_least((nvec + K - 1) / K);
    if (L > 64) continue;
    if (K > 1 && (uint64_t)L * K >= 2ull * nvec) continue;
    struct Shape { int waves, r; };
    for (Shape sh : {Shape{4, 1}, Shape{4, 2}, Shape{4, 4}, Shape{8, 1}, Shape{8, 2}}) {
      if (sh.r * K > 8) continue;                      // raw rows held in registers: at most 16 vectors
      const uint32_t groups = sh.waves * 64 / L;
      const int64_t lds_bytes = (int64_t)groups * 2 * p.cols * 4;
      if (lds_bytes > 64 * 1024) continue;
      const uint32_t tile_rows = groups * sh.r;
      const uint32_t n_tiles = (p.rows + tile_rows - 1) / tile_rows;
      uint32_t last = 0;
      for (uint32_t want : {256u, 512u, 1024u, 2048u}) {
        const uint32_t n_rb = std::min<uint32_t>(want, n_tiles);
        if (n_rb == last) continue;
        last = n_rb;
        Candidate c = make_candidate(g, "layernorm_backward", FS_SCHEME_GLOBAL, K_LAYERNORM_BWD);
        LnBwdP q = p;
        q.lanes_per_row = (int32_t)L;
        q.lanes_log2 = log2_of(L);
        q.vecs_per_lane = K;
        q.waves = sh.waves;
        q.rows_per_group = sh.r;
        q.fast = ((uint64_t)L * K == nvec && p.rows % tile_rows == 0 && n_tiles % n_rb == 0) ? 1 : 0;
        {
          Launch& l = c.launches.front();
          l.args.u.lnbwd = q;
          l.ptr[0] = in_ref(g, th);
          l.ptr[1] = in_ref(g, tdy);
          l.ptr[2] = in_ref(g, tg);
          l.ptr[3] = in_ref(g, tmu);
          l.ptr[4] = in_ref(g, trs);
          l.ptr[5] = out_ref(g.tensors[t_dx].output_slot);
          l.ptr[6] = ws_ref(0);
          l.shape.block[0] = sh.waves * 64;
          l.shape.grid[0] = n_rb;
          l.shape.lds_bytes = (uint32_t)lds_bytes;
        }
        c.launches.emplace_back();
        Launch& f = c.launches.back();
        make_fold_launch(&f, n_rb, 2 * p.cols, p.cols);
        f.ptr[0] = ws_ref(0);
        f.ptr[1] = out_ref(g.tensors[t_dg].output_slot);
        f.ptr[2] = out_ref(g.tensors[t_db].output_slot);
        c.info.n_kernels = 2;
        c.info.workspace_bytes = (int64_t)n_rb * 2 * p.cols * 4;
        c.info.lanes_per_row = (int32_t)L;
        c.info.vecs_per_lane = K;
        c.info.rows_per_block = (int32_t)tile_rows;
        c.info.lds_bytes = (int32_t)lds_bytes;
        c.info.bytes_moved_model = c.info.bytes_min + 2 * c.info.workspace_bytes;
        KernelCost kc;
        kc.hbm_bytes = 3 * n * esz + 2.0 * (double)c.info.workspace_bytes;
        kc.elems = n;
        kc.valu_per_elem = 12 + (esz == 2 ? 3 : 0);
        kc.waves_per_block = sh.waves;
        kc.waves = (double)n_rb * sh.waves;
        kc.bytes_in_flight_per_lane = 32.0 * K * sh.r;
        kc.vgpr_estimate = 24 + K * (VEC * 5 + 8 * sh.r);
        int steps = 0;
        for (uint32_t s2 = 1; s2 < L; s2 <<= 1) ++steps;
        kc.xlane_steps = 2 * steps * sh.r;
        kc.barriers = 0;
        kc.lds_bytes_per_block = (int32_t)lds_bytes;
        kc.rows_per_wave_loop = std::max(1.0, (double)n_tiles / n_rb);
        kc.dep_phases = 1;
        kc.lane_utilisation = (double)nvec / ((double)L * K);
        kc.access_run_bytes = std::min<double>(L, nvec) * 16.0;
        kc.serial_tail_s = device().mem_latency_s + 0.5 * device().launch_s + device().mem_latency_s * std::ceil(n_rb / 16.0 / 8.0) * 0.5;
        char var[56];
        snprintf(var, sizeof var, "<%s,K%d,L%u,W%d,R%d,RB%u>", dtype_name(p.dt), K, L, sh.waves, sh.r, n_rb);
        finish_candidate(&c, var, kc);
        out->push_back(c);
      }
    }
  }
  return true;
}

}  // namespace fs
