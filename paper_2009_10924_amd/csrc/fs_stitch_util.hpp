// Helpers shared by the pattern families (fs_family_*.cpp): shape predicates, buffer references and the
// bookkeeping every candidate needs.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstring>
#include <string>

#include "fs_cost.hpp"
#include "fs_internal.hpp"
#include "fs_match.hpp"

namespace fs {

inline uint32_t pow2_at_least(uint32_t v) {
  uint32_t p = 1;
  while (p < v) p <<= 1;
  return p;
}
inline int vec_of(int32_t dt) { return 16 / dtype_bytes(dt); }
inline int log2_of(uint32_t pow2) {
  int l = 0;
  while ((1u << l) < pow2) ++l;
  return l;
}

inline bool is_input(const fs_graph& g, int32_t t) { return t >= 0 && g.tensors[t].producer < 0; }
inline bool same_dims(const Tensor& a, const Tensor& b) {
  if (a.rank != b.rank) return false;
  for (int k = 0; k < a.rank; ++k)
    if (a.dims[k] != b.dims[k]) return false;
  return true;
}
// [C] or [1,..,1,C]
inline bool is_row_vector(const Tensor& v, int64_t cols) {
  if (v.dims[v.rank - 1] != cols) return false;
  for (int k = 0; k < v.rank - 1; ++k)
    if (v.dims[k] != 1) return false;
  return true;
}
inline bool covers_all(const fs_graph& g, const MatchState& st) { return st.covered.size() == g.ops.size(); }

inline BufRef in_ref(const fs_graph& g, int32_t t) {
  BufRef r;
  r.kind = BUF_INPUT;
  r.slot = g.tensors[t].input_slot;
  return r;
}
inline BufRef out_ref(int slot) {
  BufRef r;
  r.kind = BUF_OUTPUT;
  r.slot = slot;
  return r;
}
inline BufRef ws_ref(int64_t off) {
  BufRef r;
  r.kind = BUF_WORKSPACE;
  r.offset = off;
  return r;
}

inline int32_t slot_of(const fs_graph& g, int32_t t) { return t >= 0 ? g.tensors[t].input_slot : -1; }

inline Candidate make_candidate(const fs_graph& g, const char* pattern, int32_t scheme, int32_t kernel) {
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

inline void finish_candidate(Candidate* c, const char* variant, const KernelCost& cost) {
  Launch& l = c->launches.front();
  for (int k = 0; k < 3; ++k) { c->info.block[k] = (int32_t)l.shape.block[k]; c->info.grid[k] = (int32_t)l.shape.grid[k]; }
  snprintf(c->info.kernel, sizeof c->info.kernel, "%s%s", kernel_name(l.kernel), variant);
  c->cost = cost;
}

// text with every '@' replaced by `a`
inline std::string subst(const std::string& text, const std::string& a) {
  std::string r;
  for (char ch : text) {
    if (ch == '@') r += a;
    else r += ch;
  }
  return r;
}

// One pattern family: appends its candidates for `g`; returns true if it recognised the graph's shape (also when
// no compiled variant fits, in which case nothing is appended).  `pack` receives the packed form, if any.
bool build_softmax(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
bool build_layernorm(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
bool build_layernorm_backward(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
bool build_gelu(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
bool build_tchain(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
bool build_transpose(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
bool build_softmax_backward(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
bool build_rmsnorm(const fs_graph& g, std::vector<Candidate>* out, PackForm* pack);
// The launch that folds [n_rows, width] float32 column partials (second step of a global hand-off).
// K_COLFOLD over partial rows of `width` floats (`stride` floats apart, 0 = width): columns below `split` go to the
// launch's first output, the rest to its second.
void make_fold_launch(Launch* f, uint32_t n_rows, uint32_t width, uint32_t split, uint32_t stride = 0, int32_t out_dt = DT_F32);

}  // namespace fs
