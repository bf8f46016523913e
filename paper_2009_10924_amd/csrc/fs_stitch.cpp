// Stitched plans: recognise the fusion pattern, enumerate the legal schedules and
// launch dimensions for it (paper Section 4.2), and describe each one so the
// evaluator (fs_cost.cpp) can rank them.  Schedules that cannot keep a reduction row
// inside the reuse scope they rely on (one wavefront's registers, one workgroup)
// are simply not generated -- the paper's locality filter.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "fs_cost.hpp"
#include "fs_internal.hpp"
#include "fs_match.hpp"

namespace fs {

// Magic numbers for n / d, n < 2^31; checked on the spot against plain division.
FastDiv make_fastdiv(uint32_t d) {
  FastDiv f = {d == 0 ? 1u : d, 0u, 0u};
  if (d <= 1) return f;
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  f.s = l - 1;
  f.m = (uint32_t)(((1ull << (31 + l)) / d) + 1);
  const uint32_t probes[] = {0u, 1u, d - 1, d, d + 1, 2 * d - 1, 2 * d, 0x7FFFFFFFu / d * d - 1, 0x7FFFFFFFu / d * d, 0x7FFFFFFFu};
  for (uint32_t n : probes) {
    const uint32_t q = (uint32_t)(((uint64_t)n * f.m) >> 32) >> f.s;
    if (q != n / d) { f.m = 0; f.s = 0; f.d = 0; break; }   // d == 0 marks "unusable"; callers then offer no candidate
  }
  return f;
}

namespace {

uint32_t pow2_at_least(uint32_t v) {
  uint32_t p = 1;
  while (p < v) p <<= 1;
  return p;
}
int vec_of(int32_t dt) { return 16 / dtype_bytes(dt); }
int log2_of(uint32_t pow2) {
  int l = 0;
  while ((1u << l) < pow2) ++l;
  return l;
}

bool is_input(const fs_graph& g, int32_t t) { return t >= 0 && g.tensors[t].producer < 0; }
bool same_dims(const Tensor& a, const Tensor& b) {
  if (a.rank != b.rank) return false;
  for (int k = 0; k < a.rank; ++k)
    if (a.dims[k] != b.dims[k]) return false;
  return true;
}
// [C] or [1,..,1,C]
bool is_row_vector(const Tensor& v, int64_t cols) {
  if (v.dims[v.rank - 1] != cols) return false;
  for (int k = 0; k < v.rank - 1; ++k)
    if (v.dims[k] != 1) return false;
  return true;
}
bool covers_all(const fs_graph& g, const MatchState& st) { return st.covered.size() == g.ops.size(); }

BufRef in_ref(const fs_graph& g, int32_t t) {
  BufRef r;
  r.kind = BUF_INPUT;
  r.slot = g.tensors[t].input_slot;
  return r;
}
BufRef out_ref(int slot) {
  BufRef r;
  r.kind = BUF_OUTPUT;
  r.slot = slot;
  return r;
}
BufRef ws_ref(int64_t off) {
  BufRef r;
  r.kind = BUF_WORKSPACE;
  r.offset = off;
  return r;
}

int32_t slot_of(const fs_graph& g, int32_t t) { return t >= 0 ? g.tensors[t].input_slot : -1; }

Candidate make_candidate(const fs_graph& g, const char* pattern, int32_t scheme, int32_t kernel) {
  Candidate c;
  memset(&c.info, 0, sizeof c.info);
  c.info.scheme = scheme;
  c.info.n_kernels = 1;
  c.info.bytes_min = graph_bytes_min(g);
  c.info.bytes_moved_model = c.info.bytes_min;
  snprintf(c.info.pattern, sizeof c.info.pattern, "%s", pattern);
  c.launches.emplace_back();
  c.launches.back().kernel = kernel;
  return c;
}

void finish_candidate(Candidate* c, const char* variant, const KernelCost& cost) {
  Launch& l = c->launches.front();
  for (int k = 0; k < 3; ++k) { c->info.block[k] = (int32_t)l.shape.block[k]; c->info.grid[k] = (int32_t)l.shape.grid[k]; }
  snprintf(c->info.kernel, sizeof c->info.kernel, "%s%s", kernel_name(l.kernel), variant);
  c->cost = cost;
}

// ------------------------------------------------------------------ softmax family
const char* kSoftmaxTail = "div(exp(sub(@,rmax[-1](@))),rsum[-1](exp(sub(@,rmax[-1](@)))))";
std::string subst(const std::string& text, const std::string& a) {
  std::string r;
  for (char ch : text) {
    if (ch == '@') r += a;
    else r += ch;
  }
  return r;
}

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
    out->push_back(c);
  }
  return true;
}

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
  for (int K : {1, 2, 3, 4, 6, 8}) {
    const uint32_t need = (nvec + K - 1) / K;
    const uint32_t T = (need + 63) / 64 * 64;
    if (T > 256 || T < 128) continue;   // a single wave per row is the wave variant's job
    if ((uint64_t)T * K >= 2ull * nvec) continue;
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
    const uint32_t blocks_per_cu = std::max<uint32_t>(1, 2048 / T / 2);   // fill about half the wave slots per CU with one pass
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
void make_fold_launch(Launch* f, uint32_t n_rows, uint32_t width, uint32_t split) {
  f->kernel = K_COLFOLD;
  GeluP fp{};
  fp.n_row_tiles = n_rows;
  fp.cols = width;
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
  const int64_t counter_bytes = ((int64_t)n_col_tiles * 4 + 255) / 256 * 256;
  struct Shape { int waves, unroll; };
  for (int ticket = 0; ticket < 2; ++ticket) {
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
        q.ticket = ticket;
        {
          Launch& l = c.launches.front();
          l.args.u.gelu = q;
          l.ptr[0] = in_ref(g, tx);
          l.ptr[1] = in_ref(g, tb);
          l.ptr[2] = in_ref(g, tg);
          l.ptr[3] = out_ref(y.output_slot);
          l.ptr[4] = out_ref(d.output_slot);
          l.ptr[5] = ws_ref(counter_bytes);
          l.ptr[6] = ws_ref(0);
          l.shape.block[0] = sh.waves * 64;
          l.shape.grid[0] = n_rb * n_col_tiles;
        }
        if (!ticket) {
          c.launches.emplace_back();
          Launch& f = c.launches.back();
          make_fold_launch(&f, n_rb, p.cols, p.cols);
          f.ptr[0] = ws_ref(counter_bytes);
          f.ptr[1] = out_ref(d.output_slot);
          c.info.n_kernels = 2;
        }
        c.info.workspace_bytes = counter_bytes + (int64_t)n_rb * p.cols * 4;
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
        kc.barriers = ticket ? 5 : 1;
        kc.lds_bytes_per_block = c.info.lds_bytes;
        kc.rows_per_wave_loop = std::max(1.0, (double)p.rows / ((double)n_rb * tile_rows));
        kc.dep_phases = 0;   // software pipelined: only the first tile's load latency is exposed (added below)
        // the fold: a second launch spread over the chip, or one workgroup per column tile
        // reading n_rb partial rows with (threads / column quads) row groups in parallel
        if (ticket) {
          const double groups = std::max(1.0, sh.waves * 64.0 / (tile_cols / 4.0));
          kc.serial_tail_s = device().mem_latency_s * (3.0 + std::ceil(n_rb / groups / 8.0));
        } else {
          kc.serial_tail_s = device().mem_latency_s + 0.5 * device().launch_s + device().mem_latency_s * std::ceil(n_rb / 16.0 / 8.0) * 0.5;
        }
        char var[48];
        snprintf(var, sizeof var, "<%s,W%d,U%d,RB%u,%s>", dtype_name(p.dt), sh.waves, sh.unroll, n_rb, ticket ? "ticket" : "fold");
        finish_candidate(&c, var, kc);
        out->push_back(c);
      }
    }
  }
  return true;
}

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

// ------------------------------------------------------------------ generic row patterns
// A pattern served by the generic row skeleton: row inputs [.., C], column vectors [C], one output.
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
      for (uint32_t want : {512u, 1024u, 2048u}) {
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

// ------------------------------------------------------------------ lone transpose
bool build_transpose(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  if (g.ops.size() != 1 || g.ops[0].opcode != FS_TRANSPOSE || g.outputs.size() != 1) return false;
  Candidate u;
  if (build_unfused(g, &u) != FS_OK) return true;
  const Launch& l = u.launches.front();
  const bool tile = l.kernel == K_TRANSPOSE_TILE;
  u.info.scheme = tile ? FS_SCHEME_LDS : FS_SCHEME_LOCAL;
  snprintf(u.info.pattern, sizeof u.info.pattern, "transpose");
  u.info.lds_bytes = !tile ? 0 : l.args.u.transpose.vec > 1 ? 64 * 66 * l.args.u.transpose.elem_bytes : 32 * 33 * l.args.u.transpose.elem_bytes;
  KernelCost kc;
  kc.hbm_bytes = (double)u.info.bytes_min;
  kc.elems = (double)l.args.u.transpose.n;
  kc.valu_per_elem = tile ? 12 : 4;
  kc.waves_per_block = 4;
  kc.waves = (double)l.shape.grid[0] * 4;
  kc.bytes_in_flight_per_lane = tile ? (l.args.u.transpose.vec > 1 ? 64.0 * l.args.u.transpose.elem_bytes / 4.0 : 4.0 * l.args.u.transpose.elem_bytes)
                                     : (double)l.args.u.transpose.vec * l.args.u.transpose.elem_bytes;
  kc.vgpr_estimate = 24;
  kc.barriers = tile ? 1 : 0;
  kc.lds_bytes_per_block = u.info.lds_bytes;
  u.cost = kc;
  out->push_back(u);
  return true;
}

}  // namespace

std::string build_stitched(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack) {
  PackForm scratch_form;
  if (!pack) pack = &scratch_form;
  struct Family { const char* name; bool (*build)(const fs_graph&, std::vector<Candidate>*, PackForm*); };
  static const Family families[] = {
      {"softmax", build_softmax}, {"layernorm", build_layernorm}, {"bias_gelu", build_gelu},
      {"transpose_chain", build_tchain}, {"softmax_backward", build_softmax_backward}, {"rmsnorm", build_rmsnorm},
      {"layernorm_backward", build_layernorm_backward}, {"transpose", build_transpose},
  };
  std::string recognised;
  for (const Family& f : families) {
    out->clear();
    *pack = PackForm();
    if (f.build(g, out, pack)) {
      if (!out->empty()) return f.name;
      if (recognised.empty()) recognised = f.name;   // right shape of graph, but no compiled variant fits
    }
  }
  // no hand-written family: any row-local pattern still runs as one interpreted kernel
  out->clear();
  *pack = PackForm();
  if (build_row_program(g, out)) return "row_program";
  out->clear();
  return recognised;
}

}  // namespace fs
