// Structural matching of a graph against expression templates.
//
// A template is text such as
//     div(exp(sub($A,rmax[-1]($A))),rsum[-1](exp(sub($A,rmax[-1]($A)))))
// `$NAME` binds a tensor (the same name must bind the same tensor everywhere),
// `[#n]` binds the scalar attribute of scale / addc, `[-k]` on a reduction is the
// axis counted from the end, `[0213]` on tr is the permutation.  add, mul and max
// match with their operands in either order.  A match also records which ops it
// covered, so the caller can insist that the pattern is the whole graph.
#pragma once
#include <map>
#include <set>
#include <string>
#include <vector>

#include "fs_internal.hpp"

namespace fs {

struct MatchState {
  std::map<std::string, int32_t> tensors;   // $NAME -> tensor id
  std::map<int, double> scalars;            // #n -> value
  std::set<int32_t> covered;                // op indices
  int32_t convert_dtype = -1;               // dtype of a matched cvt, if any
};

class Pattern {
 public:
  explicit Pattern(const std::string& text);
  bool ok() const { return root_ >= 0; }
  // Matches the expression that produces tensor `t`; on success merges into *st.
  bool match(const fs_graph& g, int32_t t, MatchState* st) const;

 private:
  struct Node {
    bool is_var = false;
    std::string var;
    int32_t opcode = -1;
    int scalar_var = -1;        // [#n]
    bool has_axis = false;
    int axis_from_end = 0;      // negative
    std::vector<int> perm;
    int child[2] = {-1, -1};
    int n_child = 0;
  };
  std::vector<Node> nodes_;
  int root_ = -1;
  int parse(const std::string& s, size_t* pos);
  bool match_node(const fs_graph& g, int node, int32_t t, MatchState* st) const;
};

}  // namespace fs
