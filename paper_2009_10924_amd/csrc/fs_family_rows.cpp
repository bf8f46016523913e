// Pattern families on the generic row skeleton: softmax backward and RMS normalisation.
#include "fs_stitch_util.hpp"

namespace fs {

// ------------------------------------------------------------------ generic row patterns
// A pattern served by the generic row skeleton: row inputs [.., C], column vectors [C], one output.
namespace {
struct RowMatch {
  const char* name;
  int32_t pattern;
  int32_t row_in[2];      // tensor ids, -1 = unused
  int32_t vec_in[2];
  float f[4];
  double valu_per_elem;
};

void emit_row_candidates(const fs_graph& g, const RowMatch& m, std::vector<Candidate>* out, PackForm* pack) {
  const Tensor& x = g.tensors[m.row_in[0]];
  const Tensor& y = g.tensors[g.outputs[0]];
  int n_in = 0, n_vec = 0;
  for (int i = 0; i < 2; ++i) {
    if (m.row_in[i] >= 0) {
      ++n_in;
      if (!same_dims(g.tensors[m.row_in[i]], x) || g.tensors[m.row_in[i]].dtype != x.dtype) return;
    }
  }
  RowP p{};
  p.pattern = m.pattern;
  p.dt = x.dtype;
  p.cols = (uint32_t)x.dims[x.rank - 1];
  p.rows = (uint32_t)(x.numel() / p.cols);
  for (int i = 0; i < 4; ++i) p.f[i] = m.f[i];
  for (int i = 0; i < 2; ++i) {
    if (m.vec_in[i] >= 0) {
      ++n_vec;
      if (!is_row_vector(g.tensors[m.vec_in[i]], p.cols) || g.tensors[m.vec_in[i]].dtype != x.dtype) return;
    }
  }
  if (y.store_as != x.dtype || x.dtype == FS_I32 || !same_dims(y, x)) return;
  const int VEC = vec_of(p.dt);
  if (p.cols % VEC != 0) return;
  const uint32_t nvec = p.cols / VEC;
  const int esz = dtype_bytes(p.dt);
  pack->spec = m.pattern == ROW_SOFTMAX_BWD ? PACK_SOFTMAX_BWD : PACK_RMSNORM;
  pack->in_dt = pack->out_dt = p.dt;
  pack->rows = p.rows;
  pack->cols = p.cols;
  for (int i = 0; i < 4; ++i) pack->f[i] = m.f[i];
  for (int i = 0; i < 2; ++i) {
    pack->in_slot[i] = slot_of(g, m.row_in[i]);
    pack->vec_slot[i] = slot_of(g, m.vec_in[i]);
  }
  for (int K : {1, 2, 4, 8}) {
    const uint32_t L = pow2_at_least((nvec + K - 1) / K);
    if (L > 64) continue;
    if (K > 1 && (uint64_t)L * K >= 2ull * nvec) continue;
    if (K * (n_in + n_vec) > 8) continue;   // raw vectors held per lane
    Candidate c = make_candidate(g, m.name, L == 1 ? FS_SCHEME_LOCAL : FS_SCHEME_WAVE, K_ROW_WAVE);
    Launch& l = c.launches.front();
    RowP q = p;
    q.lanes_per_row = (int32_t)L;
    q.lanes_log2 = log2_of(L);
    q.vecs_per_lane = K;
    q.fast = (uint64_t)L * K == nvec && p.rows % (256 / L) == 0;
    l.args.u.row = q;
    for (int i = 0; i < 2; ++i) {
      if (m.row_in[i] >= 0) l.ptr[i] = in_ref(g, m.row_in[i]);
      if (m.vec_in[i] >= 0) l.ptr[2 + i] = in_ref(g, m.vec_in[i]);
    }
    l.ptr[4] = out_ref(0);
    l.shape.block[0] = 256;
    const uint32_t rows_per_block = 256 / L;
    l.shape.grid[0] = (p.rows + rows_per_block - 1) / rows_per_block;
    c.info.lanes_per_row = (int32_t)L;
    c.info.vecs_per_lane = K;
    c.info.rows_per_block = (int32_t)rows_per_block;
    KernelCost kc;
    kc.hbm_bytes = (n_in + 1.0) * p.rows * (double)p.cols * esz + n_vec * (double)p.cols * esz;
    kc.cache_bytes = n_vec * (double)p.rows * p.cols * esz;
    kc.elems = (double)p.rows * p.cols;
    kc.valu_per_elem = m.valu_per_elem + (esz == 2 ? 1.0 + n_in : 0.0);
    kc.waves = (double)l.shape.grid[0] * 4;
    kc.waves_per_block = 4;
    kc.bytes_in_flight_per_lane = 16.0 * K * n_in;
    kc.vgpr_estimate = 12 + K * ((n_in + n_vec) * VEC + 8);
    int steps = 0;
    for (uint32_t s = 1; s < L; s <<= 1) ++steps;
    kc.xlane_steps = steps;
    kc.lane_utilisation = (double)nvec / ((double)L * K);
    kc.access_run_bytes = std::min<double>(L, nvec) * 16.0;
    char var[48];
    snprintf(var, sizeof var, "<%s,%s,K%d,L%u>", m.name, dtype_name(p.dt), K, L);
    finish_candidate(&c, var, kc);
    out->push_back(c);
  }
  // block composition: one workgroup of T threads per row
  for (int K : {1, 2, 4}) {
    const uint32_t need = (nvec + K - 1) / K;
    const uint32_t T = (need + 63) / 64 * 64;
    if (T > 256 || T < 128) continue;
    if ((uint64_t)T * K >= 2ull * nvec) continue;
    Candidate c = make_candidate(g, m.name, FS_SCHEME_LDS, K_ROW_BLOCK);
    Launch& l = c.launches.front();
    RowP q = p;
    q.lanes_per_row = (int32_t)T;
    q.vecs_per_lane = K;
    q.fast = (uint64_t)T * K == nvec;
    l.args.u.row = q;
    for (int i = 0; i < 2; ++i) {
      if (m.row_in[i] >= 0) l.ptr[i] = in_ref(g, m.row_in[i]);
      if (m.vec_in[i] >= 0) l.ptr[2 + i] = in_ref(g, m.vec_in[i]);
    }
    l.ptr[4] = out_ref(0);
    l.shape.block[0] = T;
    l.shape.grid[0] = p.rows;
    c.info.lanes_per_row = (int32_t)T;
    c.info.vecs_per_lane = K;
    c.info.rows_per_block = 1;
    c.info.lds_bytes = 64;
    KernelCost kc;
    kc.hbm_bytes = (n_in + 1.0) * p.rows * (double)p.cols * esz + n_vec * (double)p.cols * esz;
    kc.cache_bytes = n_vec * (double)p.rows * p.cols * esz;
    kc.elems = (double)p.rows * p.cols;
    kc.valu_per_elem = m.valu_per_elem + (esz == 2 ? 1.0 + n_in : 0.0);
    kc.waves_per_block = T / 64;
    kc.waves = (double)p.rows * kc.waves_per_block;
    kc.bytes_in_flight_per_lane = 16.0 * K * n_in;
    kc.vgpr_estimate = 12 + K * ((n_in + n_vec) * VEC + 8);
    kc.xlane_steps = 6;
    kc.barriers = 1;
    kc.lds_bytes_per_block = 64;
    kc.lane_utilisation = (double)nvec / ((double)T * K);
    char var[48];
    snprintf(var, sizeof var, "<%s,%s,K%d,T%u>", m.name, dtype_name(p.dt), K, T);
    finish_candidate(&c, var, kc);
    out->push_back(c);
  }
}

}  // namespace

// dx = y * (dy - rowsum(y * dy))
bool build_softmax_backward(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  if (g.outputs.size() != 1) return false;
  Pattern pat("mul($Y,sub($DY,rsum[-1](mul($Y,$DY))))");
  MatchState st;
  if (!pat.match(g, g.outputs[0], &st) || !covers_all(g, st)) return false;
  const int32_t ty = st.tensors["Y"], tdy = st.tensors["DY"];
  if (!is_input(g, ty) || !is_input(g, tdy)) return false;
  emit_row_candidates(g, RowMatch{"softmax_backward", ROW_SOFTMAX_BWD, {ty, tdy}, {-1, -1}, {0, 0, 0, 0}, 4.0}, out, pack);
  return true;
}

// out = x * rsqrt(mean(x^2) + eps) * gamma
bool build_rmsnorm(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  if (g.outputs.size() != 1) return false;
  Pattern pat("mul(mul($X,rsqrt(addc[#0](rmean[-1](square($X))))),$G)");
  MatchState st;
  if (!pat.match(g, g.outputs[0], &st) || !covers_all(g, st)) return false;
  const int32_t tx = st.tensors["X"], tg = st.tensors["G"];
  if (!is_input(g, tx) || !is_input(g, tg)) return false;
  const Tensor& x = g.tensors[tx];
  const float inv_cols = (float)(1.0 / (double)x.dims[x.rank - 1]);
  emit_row_candidates(g, RowMatch{"rmsnorm", ROW_RMSNORM, {tx, -1}, {tg, -1}, {(float)st.scalars[0], inv_cols, 0, 0}, 5.0}, out, pack);
  return true;
}

}  // namespace fs
