// An explored program: the fusion plan of a multi-pattern graph, made executable (built by fs_explore.cpp, run by
// fs_program.cpp).
#pragma once

#include <vector>

#include "fs_internal.hpp"

extern "C" {
void fs_plan_destroy(fs_plan* p);
void fs_pack_destroy(fs_pack* p);
}

using namespace fs;

struct fs_program {
  struct Step {
    std::vector<int> ops;               // graph op indices
    double f = 0;                       // delta-evaluator gain (microseconds), 0 for a single op
    fs_plan* plan = nullptr;
    std::vector<BufRef> in, out;        // where each plan input / output lives: graph input, graph output or workspace offset
    int64_t plan_ws_offset = 0;
    int32_t pack = -1;                  // index into packs, -1 = runs on its own
    size_t own_launches = 0;            // launches of the plan issued at the step itself (the rest are joint folds)
    int32_t stage = 0;                  // external computations that must have run before it (longest chain of them)
  };
  struct JointFold { int step; size_t launch; };   // a K_COLFOLD launch of a step's plan, issued after the last step
  struct Pack {
    fs_pack* pack = nullptr;
    std::vector<int> steps;
  };
  std::vector<Step> steps;              // dependence order
  std::vector<Pack> packs;
  std::vector<std::vector<JointFold>> joint_folds;   // one launch each, at most kFoldManyMax folds in it
  fs_program_info info{};
  int32_t n_inputs = 0, n_outputs = 0;
  ~fs_program() {
    for (Step& s : steps) fs_plan_destroy(s.plan);
    for (Pack& p : packs) fs_pack_destroy(p.pack);
  }
};
