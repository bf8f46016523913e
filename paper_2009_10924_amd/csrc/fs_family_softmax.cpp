// Pattern family: row softmax with optional scale and additive mask (paper Section 4.1: warp / block composition).
#include "fs_stitch_util.hpp"

namespace fs {

// ------------------------------------------------------------------ softmax family
static const char* const kSoftmaxTail = "div(exp(sub(@,rmax[-1](@))),rsum[-1](exp(sub(@,rmax[-1](@)))))";
bool build_softmax(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  if (g.outputs.size() != 1) return false;
  static const char* pre[] = {"add(scale[#0]($X),$M)", "add($X,$M)", "scale[#0]($X)", "$X"};
  MatchState st;
  bool found = false;
  for (const char* a : pre) {
    Pattern pat(subst(kSoftmaxTail, a));
    MatchState trial;
    if (pat.match(g, g.outputs[0], &trial) && covers_all(g, trial) && is_input(g, trial.tensors["X"]) &&
        (!trial.tensors.count("M") || is_input(g, trial.tensors["M"]))) {
      st = trial;
      found = true;
      break;
    }
  }
  if (!found) return false;

  const Tensor& x = g.tensors[st.tensors["X"]];
  const Tensor& y = g.tensors[g.outputs[0]];
  const bool has_mask = st.tensors.count("M") != 0;
  SoftmaxP p{};
  p.in_dt = x.dtype;
  p.out_dt = y.store_as;
  p.cols = (uint32_t)x.dims[x.rank - 1];
  p.rows = (uint32_t)(x.numel() / p.cols);
  p.scale = st.scalars.count(0) ? (float)st.scalars[0] : 1.0f;
  p.has_mask = has_mask;
  p.ms[0] = p.ms[1] = p.ms[2] = 0;
  uint32_t od[3] = {1, 1, 1};
  for (int k = 0; k < x.rank - 1; ++k) od[3 - (x.rank - 1) + k] = (uint32_t)x.dims[k];
  bool dtype_ok = p.in_dt == p.out_dt;
  if (has_mask) {
    const Tensor& m = g.tensors[st.tensors["M"]];
    p.mask_dt = m.dtype;
    dtype_ok = dtype_ok && m.dtype == x.dtype;
    // the mask may stretch along x but must not stretch x itself
    if (!same_dims(y, x)) return true;
    int64_t acc = 1;
    for (int k = x.rank - 1; k >= 0; --k) {
      const int km = k - (x.rank - m.rank);
      const int64_t d = km >= 0 ? m.dims[km] : 1;
      const int64_t stride = d == 1 ? 0 : acc;
      acc *= d;
      if (k == x.rank - 1) p.mask_inner = d == 1 ? 0 : 1;
      else p.ms[3 - (x.rank - 1) + k] = (uint32_t)stride;
    }
  }
  if (!dtype_ok) return true;
  // neighbouring outer axes over which the mask moves alike (both stretched, or both dense) merge,
  // so the common [batch,1,1,keys] mask costs one division per row instead of two
  {
    uint32_t e[3], st[3];
    int n = 0;
    for (int k = 0; k < 3; ++k) {
      if (od[k] == 1) continue;
      if (n > 0 && ((st[n - 1] == 0 && p.ms[k] == 0) || (p.ms[k] != 0 && st[n - 1] == p.ms[k] * od[k]))) {
        e[n - 1] *= od[k];
        st[n - 1] = p.ms[k];
      } else {
        e[n] = od[k];
        st[n] = p.ms[k];
        ++n;
      }
    }
    for (int k = 0; k < 3; ++k) {
      const int src = k - (3 - n);
      od[k] = src >= 0 ? e[src] : 1;
      p.ms[k] = src >= 0 ? st[src] : 0;
    }
  }
  for (int k = 0; k < 3; ++k) {
    p.od[k] = make_fastdiv(od[k]);
    if (p.od[k].d == 0) return true;
  }

  const int VEC = vec_of(p.in_dt);
  const int esz = dtype_bytes(p.in_dt);
  const int64_t mask_bytes = has_mask ? g.tensors[st.tensors["M"]].numel() * esz : 0;
  auto base_cost = [&](KernelCost* kc) {
    kc->hbm_bytes = 2.0 * p.rows * (double)p.cols * esz + mask_bytes;
    kc->elems = (double)p.rows * p.cols;
    kc->valu_per_elem = 6.0 + (esz == 2 ? 2.0 : 0.0);
    kc->trans_per_elem = 1.0;
    kc->dep_phases = 1;
  };
  const bool vector_ok = p.cols % VEC == 0;
  const uint32_t nvec = vector_ok ? p.cols / VEC : 0;
  if (vector_ok && !has_mask) {
    pack->spec = PACK_SOFTMAX;
    pack->in_dt = pack->out_dt = p.in_dt;
    pack->rows = p.rows;
    pack->cols = p.cols;
    pack->f[0] = p.scale;
    pack->in_slot[0] = slot_of(g, st.tensors["X"]);
  }

  if (vector_ok) {
    for (int K : {1, 2, 4, 8}) {
      const uint32_t L = pow2_at_least((nvec + K - 1) / K);
      if (L > 64) continue;
      if (K > 1 && (uint64_t)L * K >= 2ull * nvec) continue;   // half the register slots would idle
      Candidate c = make_candidate(g, "softmax", L == 1 ? FS_SCHEME_LOCAL : FS_SCHEME_WAVE, K_SOFTMAX_WAVE);
      Launch& l = c.launches.front();
      SoftmaxP q = p;
      q.lanes_per_row = (int32_t)L;
      q.lanes_log2 = log2_of(L);
      q.vecs_per_lane = K;
      q.fast = (uint64_t)L * K == nvec && p.rows % (256 / L) == 0 && (!has_mask || p.mask_inner);
      l.args.u.softmax = q;
      l.ptr[0] = in_ref(g, st.tensors["X"]);
      if (has_mask) l.ptr[1] = in_ref(g, st.tensors["M"]);
      l.ptr[2] = out_ref(0);
      l.shape.block[0] = 256;
      const uint32_t rows_per_block = 256 / L;
      l.shape.grid[0] = (p.rows + rows_per_block - 1) / rows_per_block;
      c.info.lanes_per_row = (int32_t)L;
      c.info.vecs_per_lane = K;
      c.info.rows_per_block = (int32_t)rows_per_block;
      KernelCost kc;
      base_cost(&kc);
      kc.waves = (double)l.shape.grid[0] * 4;
      kc.waves_per_block = 4;
      kc.bytes_in_flight_per_lane = 16.0 * K * (has_mask && p.mask_inner ? 2 : 1);
      kc.vgpr_estimate = 12 + K * (VEC + 4) + (has_mask ? K * 4 : 0);
      int steps = 0;
      for (uint32_t s = 1; s < L; s <<= 1) ++steps;
      kc.xlane_steps = 2 * steps;
      kc.lane_utilisation = (double)nvec / ((double)L * K);
      kc.access_run_bytes = std::min<double>(L, nvec) * 16.0;
      char var[32];
      snprintf(var, sizeof var, "<%s,K%d,L%u>", dtype_name(p.in_dt), K, L);
      finish_candidate(&c, var, kc);
      out->push_back(c);
    }
    for (int K : {1, 2, 4, 8}) {
      const uint32_t need = (nvec + K - 1) / K;
      const uint32_t T = (need + 63) / 64 * 64;
      if (T > 256) continue;
      if (K > 1 && (uint64_t)T * K >= 2ull * nvec && T > 64) continue;
      if (K > 1 && T == 64 && (nvec + K / 2 - 1) / (K / 2) <= 64) continue;   // a smaller K already gives one wave
      Candidate c = make_candidate(g, "softmax", FS_SCHEME_LDS, K_SOFTMAX_BLOCK);
      Launch& l = c.launches.front();
      SoftmaxP q = p;
      q.lanes_per_row = (int32_t)T;
      q.vecs_per_lane = K;
      q.fast = (uint64_t)T * K == nvec && (!has_mask || p.mask_inner);
      l.args.u.softmax = q;
      l.ptr[0] = in_ref(g, st.tensors["X"]);
      if (has_mask) l.ptr[1] = in_ref(g, st.tensors["M"]);
      l.ptr[2] = out_ref(0);
      l.shape.block[0] = T;
      l.shape.grid[0] = p.rows;
      c.info.lanes_per_row = (int32_t)T;
      c.info.vecs_per_lane = K;
      c.info.rows_per_block = 1;
      c.info.lds_bytes = 32;
      KernelCost kc;
      base_cost(&kc);
      kc.waves_per_block = T / 64;
      kc.waves = (double)p.rows * kc.waves_per_block;
      kc.bytes_in_flight_per_lane = 16.0 * K * (has_mask && p.mask_inner ? 2 : 1);
      kc.vgpr_estimate = 16 + K * VEC + (has_mask ? VEC : 0);
      kc.xlane_steps = 12;
      kc.barriers = 2;
      kc.lds_bytes_per_block = 32;
      kc.lane_utilisation = (double)nvec / ((double)T * K);
      char var[32];
      snprintf(var, sizeof var, "<%s,K%d,T%u>", dtype_name(p.in_dt), K, T);
      finish_candidate(&c, var, kc);
      out->push_back(c);
    }
  }
  if (out->empty()) {
    // ragged or very long rows: block per row, three passes, reduced values via LDS
    Candidate c = make_candidate(g, "softmax", FS_SCHEME_LDS, K_SOFTMAX_BLOCK);
    Launch& l = c.launches.front();
    SoftmaxP q = p;
    q.lanes_per_row = 256;
    q.vecs_per_lane = 0;
    l.args.u.softmax = q;
    l.ptr[0] = in_ref(g, st.tensors["X"]);
    if (has_mask) l.ptr[1] = in_ref(g, st.tensors["M"]);
    l.ptr[2] = out_ref(0);
    l.shape.block[0] = 256;
    l.shape.grid[0] = p.rows;
    c.info.lanes_per_row = 256;
    c.info.rows_per_block = 1;
    c.info.lds_bytes = 32;
    KernelCost kc;
    base_cost(&kc);
    kc.hbm_bytes += 2.0 * p.rows * (double)p.cols * esz * 0.25;   // re-reads mostly hit L2
    kc.valu_per_elem *= 3;
    kc.trans_per_elem = 2;
    kc.dep_phases = 3;
    kc.waves_per_block = 4;
    kc.waves = (double)p.rows * 4;
    kc.bytes_in_flight_per_lane = esz;
    kc.vgpr_estimate = 24;
    kc.xlane_steps = 12;
    kc.barriers = 2;
    kc.lds_bytes_per_block = 32;
    finish_candidate(&c, "<generic>", kc);
    c.fallback = true;   // three passes over the row: passed over where a kernel generated for the row length exists
    out->push_back(c);
  }
  return true;
}

}  // namespace fs
