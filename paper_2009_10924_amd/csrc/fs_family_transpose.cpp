// Pattern families: the transpose chain (scale, row norm, permutation that keeps the innermost axis) and the lone transpose.
#include "fs_stitch_util.hpp"

namespace fs {

// ------------------------------------------------------------------ transpose chain family
bool build_tchain(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  if (g.outputs.size() != 1) return false;
  const std::string u = "mul(tr[0213]($X),$S)";
  Pattern pat("mul(" + u + ",rsqrt(addc[#0](rsum[-1](square(" + u + ")))))");
  MatchState st;
  if (!pat.match(g, g.outputs[0], &st) || !covers_all(g, st)) return false;
  int32_t tx = st.tensors["X"], ts = st.tensors["S"];
  if (!is_input(g, tx) || !is_input(g, ts)) return false;
  const Tensor& x = g.tensors[tx];
  const Tensor& s = g.tensors[ts];
  if (x.rank != 4) return true;
  TChainP p{};
  p.B = (uint32_t)x.dims[0]; p.S = (uint32_t)x.dims[1]; p.H = (uint32_t)x.dims[2]; p.D = (uint32_t)x.dims[3];
  // scale must be one value per head: [H,1,1] (or [1,H,1,1])
  if (s.numel() != (int64_t)p.H || s.rank < 3 || s.dims[s.rank - 3] != (int64_t)p.H) return true;
  p.dt = x.dtype;
  p.scale_dt = s.dtype;
  p.eps = (float)st.scalars[0];
  if (s.dtype != x.dtype || g.tensors[g.outputs[0]].store_as != x.dtype) return true;
  const int VEC = vec_of(p.dt);
  if (p.D % VEC != 0) return true;
  const uint32_t nvec = p.D / VEC;
  const int esz = dtype_bytes(p.dt);
  const double n = (double)x.numel();

  for (int lds = 0; lds < 2; ++lds) {
    for (int K : {1, 2, 4}) {
      const uint32_t L = pow2_at_least((nvec + K - 1) / K);
      if (L > 64) continue;
      if (K > 1 && (uint64_t)L * K >= 2ull * nvec) continue;
      const uint32_t groups = 256 / L;
      for (uint32_t s_tile : {1u, 2u, 3u, 4u, 6u, 8u, 12u, 16u}) {
        if (s_tile > 1 && s_tile >= 2 * p.S) continue;
        const uint32_t tile_rows = s_tile * p.H;
        const uint32_t passes = (tile_rows + groups - 1) / groups;
        if (passes > 4 || passes * K > 8) continue;
        if ((double)tile_rows / (passes * groups) < 0.7 && s_tile > 1) continue;   // too many idle lane groups
        const int64_t lds_bytes = lds ? (int64_t)tile_rows * (p.D + 4) * 4 : 0;
        if (lds_bytes > 64 * 1024) continue;
        Candidate c = make_candidate(g, "transpose_chain", lds ? FS_SCHEME_LDS : (L == 1 ? FS_SCHEME_LOCAL : FS_SCHEME_WAVE),
                                     lds ? K_TCHAIN_LDS : K_TCHAIN_WAVE);
        Launch& l = c.launches.front();
        TChainP q = p;
        q.lanes_per_row = (int32_t)L;
        q.lanes_log2 = log2_of(L);
        q.vecs_per_lane = K;
        q.s_tile = (int32_t)s_tile;
        q.passes = (int32_t)passes;
        q.div_h = make_fastdiv(p.H);
        q.div_s_tiles = make_fastdiv((p.S + s_tile - 1) / s_tile);
        if (q.div_h.d == 0 || q.div_s_tiles.d == 0) continue;
        l.args.u.tchain = q;
        l.ptr[0] = in_ref(g, tx);
        l.ptr[1] = in_ref(g, ts);
        l.ptr[2] = out_ref(0);
        l.shape.block[0] = 256;
        l.shape.grid[0] = p.B * ((p.S + s_tile - 1) / s_tile);
        l.shape.lds_bytes = (uint32_t)lds_bytes;
        c.info.lanes_per_row = (int32_t)L;
        c.info.vecs_per_lane = K;
        c.info.rows_per_block = (int32_t)tile_rows;
        c.info.lds_bytes = (int32_t)lds_bytes;
        KernelCost kc;
        kc.hbm_bytes = 2 * n * esz;
        kc.elems = n;
        kc.valu_per_elem = 5 + (esz == 2 ? 2 : 0) + (lds ? 2 : 0);
        kc.trans_per_elem = 0;
        kc.waves_per_block = 4;
        kc.waves = (double)l.shape.grid[0] * 4;
        kc.rows_per_wave_loop = 1;
        kc.bytes_in_flight_per_lane = 16.0 * K * passes;
        kc.vgpr_estimate = 16 + K * VEC * (int)passes * 2;
        int steps = 0;
        for (uint32_t t = 1; t < L; t <<= 1) ++steps;
        kc.xlane_steps = steps * (int)passes;
        kc.barriers = lds ? 1 : 0;
        kc.lds_bytes_per_block = (int32_t)lds_bytes;
        kc.lds_traffic_bytes = lds ? 2 * n * 4 : 0;
        kc.store_run_bytes = lds ? (double)s_tile * p.D * esz : (double)p.D * esz;
        kc.lane_utilisation = (double)nvec / ((double)L * K) * (double)tile_rows / (passes * groups);
        kc.access_run_bytes = std::min<double>(L, nvec) * 16.0;
        char var[48];
        snprintf(var, sizeof var, "<%s,K%d,L%u,S%u,P%u>", dtype_name(p.dt), K, L, s_tile, passes);
        finish_candidate(&c, var, kc);
        out->push_back(c);
      }
    }
  }
  return true;
}

// ------------------------------------------------------------------ lone transpose
bool build_transpose(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  if (g.ops.size() != 1 || g.ops[0].opcode != FS_TRANSPOSE || g.outputs.size() != 1) return false;
  Candidate u;
  if (build_unfused(g, &u) != FS_OK) return true;
  const Launch& l = u.launches.front();
  const bool tile = l.kernel == K_TRANSPOSE_TILE;
  u.info.scheme = tile ? FS_SCHEME_LDS : FS_SCHEME_LOCAL;
  snprintf(u.info.pattern, sizeof u.info.pattern, "transpose");
  u.info.lds_bytes = !tile ? 0 : l.args.u.transpose.vec > 1 ? 256 * 16 * l.args.u.transpose.vec : 32 * 33 * l.args.u.transpose.elem_bytes;
  KernelCost kc;
  kc.hbm_bytes = (double)u.info.bytes_min;
  kc.elems = (double)l.args.u.transpose.n;
  kc.valu_per_elem = tile ? 12 : 4;
  kc.waves_per_block = 4;
  kc.waves = (double)l.shape.grid[0] * 4;
  kc.bytes_in_flight_per_lane = tile ? (l.args.u.transpose.vec > 1 ? 16.0 * l.args.u.transpose.vec : 4.0 * l.args.u.transpose.elem_bytes)
                                     : (double)l.args.u.transpose.vec * l.args.u.transpose.elem_bytes;
  kc.vgpr_estimate = 24;
  kc.barriers = tile ? 1 : 0;
  kc.lds_bytes_per_block = u.info.lds_bytes;
  u.cost = kc;
  out->push_back(u);
  return true;
}

}  // namespace fs
