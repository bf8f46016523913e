// Stitched plans: recognise the fusion pattern, enumerate the legal schedules and
// launch dimensions for it (paper Section 4.2), and describe each one so the
// evaluator (fs_cost.cpp) can rank them.  Schedules that cannot keep a reduction row
// inside the reuse scope they rely on (one wavefront's registers, one workgroup)
// are simply not generated -- the paper's locality filter.
#include "fs_stitch_util.hpp"

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
      if (!out->empty()) {
        // a family that only has its slow catch-all kernel for these extents (ragged or very long rows): the row
        // program's candidates join the list, and the choice passes the catch-all over while one of them stands
        bool only_fallbacks = true;
        for (const Candidate& c : *out) only_fallbacks = only_fallbacks && c.fallback;
        if (only_fallbacks) {
          std::vector<Candidate> more;
          if (build_row_program(g, &more)) out->insert(out->end(), more.begin(), more.end());
        }
        return f.name;
      }
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
